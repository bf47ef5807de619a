// Decode attention, plain-VALU variant, and the split-K merge kernel.
//
// One workgroup (4 waves) per item of a (query, kv-head); items are dealt by size and take static
// shares of the page lists.  A wave takes every fourth page of the item.  For a page it dequantises K in binary32 straight from the packed chunks (lane (j,t)
// owns slot t, channels 32g+8j..+7 of every group g), reduces the partial dot products over the
// four j lanes, updates the running softmax, then walks the V chunks (lane (q,m) owns slots
// 4q..4q+3, channels 16mb+m).  It is the simple, easily checked path; the MFMA kernel in
// decode_mfma.hip is the fast one and must agree with it.
#include "decode_common.h"

namespace thinkv {

__device__ inline uint32_t field(const uint32_t* w, int f, int h, int bits) {
  const int fph = 16 / bits;
  return (w[f / fph] >> (16 * h + bits * (f % fph))) & ((1u << bits) - 1u);
}

template <int D>
__global__ __launch_bounds__(256) void decode_simple_kernel(thinkv_view v, DecodeArgs a) {
  constexpr int NG = D / kGroup, NM = D / 16, GMAX = 8;
  const thinkv_config& c = v.cfg;
  const ItemLoc it = locate_item(v, a, blockIdx.x);
  if (it.j >= it.n) return;
  const int b = it.b, hkv = it.hkv;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int Hq = c.n_q_heads, H = c.n_kv_heads, G = Hq / H;
  const int seq = a.seq_ids[b];
  __shared__ float s_q[GMAX][D];
  __shared__ float s_m[4][GMAX], s_l[4][GMAX];
  __shared__ float s_acc[4][GMAX][D];

  int np[3];
  seq_pages(v, a.layer, seq, np);
  if (it.j == 0 && tid == 0) {
    a.alloc[2 * (b * H + hkv)] = it.row0;
    a.alloc[2 * (b * H + hkv) + 1] = it.n;
  }
  for (int i = tid; i < G * D; i += 256)
    s_q[i / D][i % D] = load_as_f32(a.q, ((int64_t)b * Hq + hkv * G) * D + i, a.q_dtype) * a.scale_log2e;
  __syncthreads();

  const int j = lane >> 4, t = lane & 15;   // K view: octet j, slot t
  const int vq = lane >> 4, vm = lane & 15; // V view: slot quad vq, channel vm of every block
  float m_run[GMAX], l_run[GMAX], acc[GMAX][NM];
  for (int g = 0; g < GMAX; ++g) {
    m_run[g] = -INFINITY;
    l_run[g] = 0.f;
    for (int mb = 0; mb < NM; ++mb) acc[g][mb] = 0.f;
  }
  const int qpos = a.window > 0 ? a.q_pos[b] : 0;

  for (int k = 0; k < 3; ++k) {
    const int bits = c.bits_of_class[k];
    const bool fp = c.format == THINKV_FMT_FP;
    const BlockGeom geo = block_geom(bits, D, c.format);
    const int p0 = (int)((int64_t)it.j * np[k] / it.n), p1 = (int)((int64_t)(it.j + 1) * np[k] / it.n);
    const int32_t* tab = v.block_table + table_base(c, seq, a.layer, k);
    const uint32_t* msk = v.slot_mask + table_base(c, seq, a.layer, k);
    for (int pi = p0 + wave; pi < p1; pi += 4) {
      const int pid = tab[pi];
      uint32_t live = msk[pi] & 0xFFFFu;
      if (a.window > 0) {
        const int sp = v.slot_pos[k][(int64_t)pid * kPage + t];
        const int d = qpos - sp;
        const bool vis = d >= 0 && d < a.window;
        live &= (uint32_t)(__ballot(vis) & 0xFFFFull);
      }
      if (live == 0) continue;
      const uint8_t* blk = v.arena[k] + ((int64_t)pid * H + hkv) * geo.block_bytes;
      // ---- scores
      uint32_t kw[8];
      const uint32_t* kc = (const uint32_t*)(blk + geo.k_codes + lane * geo.chunk_bytes);
      for (int w = 0; w < geo.chunk_bytes / 4; ++w) kw[w] = kc[w];
      const _Float16* kmeta = (const _Float16*)(blk + geo.k_meta);
      float part[GMAX];
      for (int g = 0; g < GMAX; ++g) part[g] = 0.f;
      for (int grp = 0; grp < NG; ++grp) {
        float sc, zp = 0.f;
        if (fp) {
          // channels 32 grp + 8 j .. + 7 lie in the group of 16 number 2 grp + j / 2
          sc = bits == 8 ? c.fp8_scale[0] : e4m3_value(((const uint8_t*)kmeta)[(2 * grp + (j >> 1)) * kPage + t]);
        } else {
          sc = (float)kmeta[meta_index(t, grp)];
          zp = (float)kmeta[meta_index(t, grp) + 4];
        }
        for (int e = 0; e < 8; ++e) {
          const uint32_t code = field(kw, 4 * grp + (e >> 1), e & 1, bits);
          const float kh = fp ? fp_code_value(code, bits) * sc : fmaf((float)code, sc, zp);
          const int ch = 32 * grp + 8 * j + e;
          for (int g = 0; g < GMAX; ++g)
            if (g < G) part[g] = fmaf(kh, s_q[g][ch], part[g]);
        }
      }
      const bool alive = (live >> t) & 1u;
      float p[GMAX];
      for (int g = 0; g < GMAX; ++g) {
        if (g >= G) { p[g] = 0.f; continue; }
        float s = part[g];
        s += __shfl_xor(s, 16, 64);
        s += __shfl_xor(s, 32, 64);
        s = alive ? s : -INFINITY;
        float mx = s;
        for (int d = 8; d >= 1; d >>= 1) mx = fmaxf(mx, __shfl_xor(mx, d, 64));
        const float m_new = fmaxf(m_run[g], mx);  // finite: the page has a live slot
        const float corr = exp2f(m_run[g] - m_new);
        p[g] = exp2f(s - m_new);
        float ps = p[g];
        for (int d = 8; d >= 1; d >>= 1) ps += __shfl_xor(ps, d, 64);
        l_run[g] = l_run[g] * corr + ps;
        m_run[g] = m_new;
        for (int mb = 0; mb < NM; ++mb) acc[g][mb] *= corr;
      }
      // ---- values
      uint32_t vw[8];
      const uint32_t* vc = (const uint32_t*)(blk + geo.v_codes + lane * geo.chunk_bytes);
      for (int w = 0; w < geo.chunk_bytes / 4; ++w) vw[w] = vc[w];
      const _Float16* vmeta = (const _Float16*)(blk + geo.v_meta);
      for (int r = 0; r < 4; ++r) {
        const int tok = 4 * vq + r;
        float pr[GMAX];
        for (int g = 0; g < GMAX; ++g) pr[g] = (g < G) ? __shfl(p[g], tok, 64) : 0.f;
        for (int mb = 0; mb < NM; ++mb) {
          float sc, zp = 0.f;
          if (fp) {   // channel block mb is a group of 16
            sc = bits == 8 ? c.fp8_scale[1] : e4m3_value(((const uint8_t*)vmeta)[mb * kPage + tok]);
          } else {
            sc = (float)vmeta[meta_index(tok, mb >> 1)];
            zp = (float)vmeta[meta_index(tok, mb >> 1) + 4];
          }
          const uint32_t code = field(vw, (r >> 1) * NM + mb, r & 1, bits);
          const float vh = fp ? fp_code_value(code, bits) * sc : fmaf((float)code, sc, zp);
          for (int g = 0; g < GMAX; ++g)
            if (g < G) acc[g][mb] = fmaf(pr[g], vh, acc[g][mb]);
        }
      }
    }
  }
  // ---- fold the four slot quads, then the four waves
  for (int g = 0; g < GMAX; ++g) {
    if (g >= G) continue;
    for (int mb = 0; mb < NM; ++mb) {
      float x = acc[g][mb];
      x += __shfl_xor(x, 16, 64);
      x += __shfl_xor(x, 32, 64);
      if (vq == 0) s_acc[wave][g][16 * mb + vm] = x;
    }
    if (lane == 0) {
      s_m[wave][g] = m_run[g];
      s_l[wave][g] = l_run[g];
    }
  }
  __syncthreads();
  for (int i = tid; i < G * D; i += 256) {
    const int g = i / D, ch = i % D;
    float M = -INFINITY;
    for (int w = 0; w < 4; ++w) M = fmaxf(M, s_m[w][g]);
    float L = 0.f, A = 0.f;
    for (int w = 0; w < 4; ++w) {
      const float f = (s_m[w][g] == -INFINITY) ? 0.f : exp2f(s_m[w][g] - M);
      L += s_l[w][g] * f;
      A += s_acc[w][g][ch] * f;
    }
    float* dst = partial_row(a, G, D, it.row0 + it.j, g);
    dst[ch] = A;
    if (ch == 0) {
      dst[D] = M;
      dst[D + 1] = L;
    }
  }
}

// One workgroup of D threads per (query, query head): log-sum-exp merge of the head's partial rows
// (first row and count as item 0 of the head left them).  Maxima and weights are found with one
// row per thread; the weighted sum over rows is unrolled so that several rows are in flight per thread.
template <int D>
__global__ __launch_bounds__(D) void decode_merge_kernel(thinkv_view v, DecodeArgs a) {
  const thinkv_config& c = v.cfg;
  const int hq = blockIdx.x, b = blockIdx.y, ch = threadIdx.x;
  const int Hq = c.n_q_heads, G = Hq / c.n_kv_heads, hkv = hq / G;
  __shared__ float s_w[kMaxRowsPerHead];
  __shared__ float s_red[D / 64];
  const int row0 = a.alloc[2 * (b * c.n_kv_heads + hkv)];
  int ns = a.alloc[2 * (b * c.n_kv_heads + hkv) + 1];
  ns = ns > kMaxRowsPerHead ? kMaxRowsPerHead : ns;
  constexpr int RS = D + kRowPad;
  const float* src = partial_row(a, G, D, row0, hq % G);
  const int64_t stride = (int64_t)G * RS;   // from one row of this query head to the next
  // maximum over rows
  float m_loc = -INFINITY;
  for (int s = ch; s < ns; s += D) {
    const float m = src[s * stride + D];
    s_w[s] = m;
    m_loc = fmaxf(m_loc, m);
  }
  for (int d = 32; d >= 1; d >>= 1) m_loc = fmaxf(m_loc, __shfl_xor(m_loc, d, 64));
  if ((ch & 63) == 0) s_red[ch >> 6] = m_loc;
  __syncthreads();
  float M = s_red[0];
  for (int w = 1; w < D / 64; ++w) M = fmaxf(M, s_red[w]);
  __syncthreads();
  // weights and denominator
  float l_loc = 0.f;
  for (int s = ch; s < ns; s += D) {
    const float m = s_w[s];
    const float f = (m == -INFINITY) ? 0.f : exp2f(m - M);
    s_w[s] = f;
    l_loc = fmaf(src[s * stride + D + 1], f, l_loc);
  }
  for (int d = 32; d >= 1; d >>= 1) l_loc += __shfl_xor(l_loc, d, 64);
  if ((ch & 63) == 0) s_red[ch >> 6] = l_loc;
  __syncthreads();
  float L = s_red[0];
  for (int w = 1; w < D / 64; ++w) L += s_red[w];
  // weighted sum of the partial rows
  float A = 0.f;
  const float* col = src + ch;
  int s = 0;
  for (; s + 4 <= ns; s += 4) {
    const float x0 = col[(s + 0) * stride], x1 = col[(s + 1) * stride];
    const float x2 = col[(s + 2) * stride], x3 = col[(s + 3) * stride];
    A = fmaf(x0, s_w[s], A);
    A = fmaf(x1, s_w[s + 1], A);
    A = fmaf(x2, s_w[s + 2], A);
    A = fmaf(x3, s_w[s + 3], A);
  }
  for (; s < ns; ++s) A = fmaf(col[s * stride], s_w[s], A);
  // the work queues of this (query, kv-head) are left empty for the next call
  if (ch < 4 && hq % G == 0 && b < c.max_seqs)
    v.work_counters[(((int64_t)a.layer * c.max_seqs + b) * c.n_kv_heads + hkv) * 4 + ch] = 0u;
  const float o = L > 0.f ? A / L : 0.f;
  store_from_f32(a.out, ((int64_t)b * Hq + hq) * D + ch, a.out_dtype, o);
  if (a.lse && ch == 0) a.lse[(int64_t)b * Hq + hq] = L > 0.f ? (M + log2f(L)) * 0.6931471805599453f : -INFINITY;
}

int launch_decode_simple(const thinkv_view& v, const DecodeArgs& a, hipStream_t st) {
  dim3 grid(a.n_rows);
  if (v.cfg.head_dim == 128)
    hipLaunchKernelGGL(decode_simple_kernel<128>, grid, dim3(256), 0, st, v, a);
  else
    hipLaunchKernelGGL(decode_simple_kernel<64>, grid, dim3(256), 0, st, v, a);
  return hipGetLastError() == hipSuccess ? THINKV_OK : THINKV_E_HIP;
}

int launch_decode_merge(const thinkv_view& v, const DecodeArgs& a, hipStream_t st) {
  dim3 grid(v.cfg.n_q_heads, a.B);
  if (v.cfg.head_dim == 128)
    hipLaunchKernelGGL(decode_merge_kernel<128>, grid, dim3(128), 0, st, v, a);
  else
    hipLaunchKernelGGL(decode_merge_kernel<64>, grid, dim3(64), 0, st, v, a);
  return hipGetLastError() == hipSuccess ? THINKV_OK : THINKV_E_HIP;
}

}  // namespace thinkv
