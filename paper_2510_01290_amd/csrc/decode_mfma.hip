// Decode attention on the matrix cores (gfx950).
//
// The affine dequantisation is distributed over the dot products so that the matrix cores
// only ever see exact operands:
//
//   scores   q.k^_t = sum_g [ s_K(t,g) * (sum_{i in g} q_i c_K(t,i)) + zp_K(t,g) * (sum_{i in g} q_i) ]
//   values   o_c    = sum_t [ (p_t s_V(t,g(c))) * c_V(t,c) ]  +  sum_t p_t zp_V(t,g(c))
//
// The integer codes c are fed to v_mfma_f32_16x16x32_f16 as binary16 numbers without any
// conversion: a b-bit field masked inside a 16-bit half IS the binary16 (sub)normal
// c * 2^(position-24); the power of two is folded into the query (for K) or into the output
// scale (for V).  A quantisation group is 32 channels = the K extent of one MFMA, so group
// scales multiply whole MFMA results in binary32.  Scores are computed transposed
// (tokens x heads) so that their register layout is already the B-operand layout of the PV
// product; the 16 MFMA columns carry the G query heads of the group, a duplicate of them
// that takes the low half of a two-term binary16 split of p*s_V (22 significant bits), and
// padding.  Per-token scales reach the lanes that need them through DPP row broadcasts.
//
// One workgroup of four waves per (query, kv-head, item); an item holds pages of one thought
// type, so the bit width is a compile-time constant of the inner loop; a wave walks every
// fourth page pair of the item; the four waves are merged through LDS into one partial
// (m, l, acc) per query head.
#include "decode_common.h"

namespace thinkv {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half2v __attribute__((ext_vector_type(2)));
typedef float float4v __attribute__((ext_vector_type(4)));
typedef float float2v __attribute__((ext_vector_type(2)));
typedef uint32_t uint4v __attribute__((ext_vector_type(4)));

union H8 {
  half8 h;
  uint32_t u[4];
};

template <int N>
__device__ __forceinline__ float bcast_row(float v) {
  // value of lane N of this lane's row of 16
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x150 + N, 0xf, 0xf, true));
}

__device__ __forceinline__ uint32_t pack_rne(float a, float b) {
  float2v f = {a, b};
  half2v h = __builtin_convertvector(f, half2v);
  return __builtin_bit_cast(uint32_t, h);
}

__device__ __forceinline__ float half_lo(uint32_t u) { return (float)__builtin_bit_cast(_Float16, (uint16_t)(u & 0xFFFFu)); }
__device__ __forceinline__ float half_hi(uint32_t u) { return (float)__builtin_bit_cast(_Float16, (uint16_t)(u >> 16)); }

// Field geometry of a b-bit layout: FPH fields per 16-bit half-word.  The matrix core adds the
// products of one instruction in a fixed-width window below the largest *nominal* product
// exponent, and a subnormal operand keeps its nominal exponent (2^-14) however many leading
// zeros it has -- so a code left at the bottom of the half-word would cost up to ten bits of the
// sum.  Every field is therefore moved, by one shift shared with its neighbour field, to sit
// just under bit 11 (offset OMIN or OMIN + BITS), and only the residual 2^REL is folded into
// the other operand.  8-bit codes fill the low byte as they are.
template <int BITS>
struct Fld {
  static constexpr int FPH = 16 / BITS;
  static constexpr uint32_t MASK = ((1u << BITS) - 1u) * 0x00010001u;
  static constexpr int OMIN = BITS == 2 ? 7 : (BITS == 4 ? 3 : 0);
  __device__ static constexpr int rel_of(int f) { return BITS == 8 ? 0 : BITS * ((f % FPH) & 1); }
  // operand register (two codes: low/high half) for field f of the chunk words w[]
  __device__ static __forceinline__ uint32_t get(const uint32_t* w, int f) {
    const int word = f / FPH, pos = f % FPH;
    const uint32_t x = w[word];
    if constexpr (BITS == 8) {
      return (pos == 0 ? x : (x >> 8)) & MASK;
    } else {
      // field pair (pos & ~1, pos | 1) starts at bit BITS*(pos & ~1); bring it to bit OMIN
      const int from = BITS * (pos & ~1);
      const uint32_t y = from <= OMIN ? (x << (OMIN - from)) : (x >> (from - OMIN));
      return y & (MASK << (OMIN + BITS * (pos & 1)));
    }
  }
};

template <int D, int BITS>
struct PageRegs {
  static constexpr int CW = (D / 32) * BITS / 4;  // chunk dwords
  uint32_t kw[CW], vw[CW];
  uint32_t kmeta, vmeta;
};

template <int D, int BITS>
__device__ __forceinline__ void load_page(PageRegs<D, BITS>& r, const uint8_t* blk, int lane, int meta_idx) {
  constexpr int CW = PageRegs<D, BITS>::CW;
  const BlockGeom g = block_geom(BITS, D);
  const uint32_t* kc = (const uint32_t*)(blk + g.k_codes) + lane * CW;
  const uint32_t* vc = (const uint32_t*)(blk + g.v_codes) + lane * CW;
  if constexpr (CW == 1) {
    r.kw[0] = kc[0];
    r.vw[0] = vc[0];
  } else if constexpr (CW == 2) {
    const uint2 a = *(const uint2*)kc, b = *(const uint2*)vc;
    r.kw[0] = a.x; r.kw[1] = a.y;
    r.vw[0] = b.x; r.vw[1] = b.y;
  } else {
#pragma unroll
    for (int i = 0; i < CW; i += 4) {
      const uint4 a = *(const uint4*)(kc + i), b = *(const uint4*)(vc + i);
      r.kw[i] = a.x; r.kw[i + 1] = a.y; r.kw[i + 2] = a.z; r.kw[i + 3] = a.w;
      r.vw[i] = b.x; r.vw[i + 1] = b.y; r.vw[i + 2] = b.z; r.vw[i + 3] = b.w;
    }
  }
  r.kmeta = ((const uint32_t*)(blk + g.k_meta))[meta_idx];
  r.vmeta = ((const uint32_t*)(blk + g.v_meta))[meta_idx];
}

template <int D>
struct WaveState {
  static constexpr int NG = D / 32, NM = D / 16;
  float4v o[NM];   // o[mb][r]: channel 16*mb + 4*q + r, column n
  float ozp[NG];   // zero-point part of the output, this lane's own tokens only
  float m, l;      // running maximum (log2 domain) of column n; partial sum of p over own tokens
};

// maximum over the four lanes that share a column (lane ^ 16, lane ^ 32), on the VALU
__device__ __forceinline__ float col_max(float x) {
  const uint32_t u = __builtin_bit_cast(uint32_t, x);
  auto r16 = __builtin_amdgcn_permlane16_swap(u, u, false, false);   // rows (0,1) and (2,3) exchanged
  x = fmaxf(__builtin_bit_cast(float, (uint32_t)r16[0]), __builtin_bit_cast(float, (uint32_t)r16[1]));
  const uint32_t w = __builtin_bit_cast(uint32_t, x);
  auto r32 = __builtin_amdgcn_permlane32_swap(w, w, false, false);   // halves exchanged
  return fmaxf(__builtin_bit_cast(float, (uint32_t)r32[0]), __builtin_bit_cast(float, (uint32_t)r32[1]));
}

struct PairIds {
  int pid_a, pid_b;
  uint32_t live_a, live_b;
};

template <int D, int BITS>
struct PairRegs {
  PageRegs<D, BITS> a, b;
};

// One class (bit width) of one wave's share of the item: page pairs wave, wave+4, ... of
// tab[p0..p1).
template <int D, int BITS, int G>
struct ClassRunner {
  static constexpr int NG = D / 32, NM = D / 16;
  using F = Fld<BITS>;
  WaveState<D>& st;
  const thinkv_view& v;
  const DecodeArgs& a;
  const int cls, hkv, qpos;
  const int32_t* tab;
  const int p0, p1, wave;
  int lane, qd, n;
  float alpha;
  H8 bq[NG];
  float qsum[NG];

  __device__ __forceinline__ ClassRunner(WaveState<D>& st_, const thinkv_view& v_, const DecodeArgs& a_, int cls_, const int32_t* tab_,
                                         int p0_, int p1_, int wave_, int hkv_, const _Float16* s_q, const float* s_qsum, int qpos_)
      : st(st_), v(v_), a(a_), cls(cls_), hkv(hkv_), qpos(qpos_), tab(tab_), p0(p0_), p1(p1_), wave(wave_) {
    lane = threadIdx.x & 63;
    qd = lane >> 4;
    n = lane & 15;
    alpha = (n >= G && n < 2 * G) ? 1.0f : 0.0f;
    // B operand of the score product for this bit width: q of column n, channels (g, 8qd+e),
    // scaled down by the residual power of two its code carries
    const int head = n < G ? n : n - G;
#pragma unroll
    for (int g = 0; g < NG; ++g) {
      qsum[g] = n < 2 * G ? s_qsum[head * NG + g] : 0.f;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const int f = 4 * g + (e >> 1);
        float x = n < 2 * G ? (float)s_q[head * D + 32 * g + 8 * qd + e] : 0.f;
        x *= 1.0f / (float)(1 << F::rel_of(f));
        bq[g].h[e] = (_Float16)x;   // exact: power-of-two scaling of a binary16 value
      }
    }
  }

  __device__ __forceinline__ void issue_loads(PairRegs<D, BITS>& r, const PairIds& id) const {
    if ((id.live_a | id.live_b) == 0) return;
    const int H = v.cfg.n_kv_heads;
    const BlockGeom geo = block_geom(BITS, D);
    const uint8_t* blk_a = v.arena[cls] + ((int64_t)id.pid_a * H + hkv) * geo.block_bytes;
    const uint8_t* blk_b = v.arena[cls] + ((int64_t)id.pid_b * H + hkv) * geo.block_bytes;
    if constexpr (D == 128) {
      load_page<D, BITS>(r.a, blk_a, lane, lane);
      load_page<D, BITS>(r.b, blk_b, lane, lane);
    } else {
      // 32 meta dwords per page: lanes x<8 of every row take page a, x>=8 page b
      const int mi = 8 * qd + (n & 7);
      load_page<D, BITS>(r.a, blk_a, lane, mi);
      load_page<D, BITS>(r.b, blk_b, lane, mi);
    }
  }

  __device__ __forceinline__ void compute(const PairRegs<D, BITS>& r, const PairIds& id) {
    const uint32_t live_a = id.live_a, live_b = id.live_b;
    if ((live_a | live_b) == 0) return;
    const PageRegs<D, BITS>& ra = r.a;
    const PageRegs<D, BITS>& rb = r.b;
    uint32_t kma = ra.kmeta, vma = ra.vmeta;
    if constexpr (D == 64) {
      if (n >= 8) { kma = rb.kmeta; vma = rb.vmeta; }
    }
    // per-lane converted meta: scale (times the power of two the codes lack) and zero-point
    constexpr float KS = (float)(1 << (24 - F::OMIN));   // codes enter the MFMA as c * 2^(OMIN - 24)
    const float ks_a = half_lo(kma) * KS, kz_a = half_hi(kma);
    const float vs_a = half_lo(vma), vz_a = half_hi(vma);
    float ks_b = ks_a, kz_b = kz_a, vs_b = vs_a, vz_b = vz_a;
    if constexpr (D == 128) {
      ks_b = half_lo(rb.kmeta) * KS; kz_b = half_hi(rb.kmeta);
      vs_b = half_lo(rb.vmeta); vz_b = half_hi(rb.vmeta);
    }

    // ---------------- scores: S^T[token][column] per page
    float sa[4], sb[4];
#pragma unroll
    for (int r4 = 0; r4 < 4; ++r4) sa[r4] = sb[r4] = 0.f;
#pragma unroll
    for (int g = 0; g < NG; ++g) {
      H8 ka, kb;
#pragma unroll
      for (int vv = 0; vv < 4; ++vv) {
        ka.u[vv] = F::get(ra.kw, 4 * g + vv);
        kb.u[vv] = F::get(rb.kw, 4 * g + vv);
      }
      const float4v z = {0.f, 0.f, 0.f, 0.f};
      const float4v ya = __builtin_amdgcn_mfma_f32_16x16x32_f16(ka.h, bq[g].h, z, 0, 0, 0);
      const float4v yb = __builtin_amdgcn_mfma_f32_16x16x32_f16(kb.h, bq[g].h, z, 0, 0, 0);
      // scale/zero-point of (token 4qd+r, group g) sit in lane 4r+g of this row (D=128),
      // or lane 8p+2r+g (D=64, p = page)
#define TKV_SCORE_STEP(R)                                                                              \
  {                                                                                                    \
    constexpr int IA = (D == 128) ? (4 * R + GI) : (2 * R + GI);                                        \
    constexpr int IB = (D == 128) ? (4 * R + GI) : (8 + 2 * R + GI);                                    \
    sa[R] = fmaf(bcast_row<IA>(ks_a), ya[R], sa[R]);                                                   \
    sa[R] = fmaf(bcast_row<IA>(kz_a), qsum[g], sa[R]);                                                 \
    sb[R] = fmaf(bcast_row<IB>(D == 128 ? ks_b : ks_a), yb[R], sb[R]);                                 \
    sb[R] = fmaf(bcast_row<IB>(D == 128 ? kz_b : kz_a), qsum[g], sb[R]);                               \
  }
#define TKV_SCORE_GROUP(GI_)            \
  if (g == GI_) {                       \
    constexpr int GI = GI_;             \
    TKV_SCORE_STEP(0) TKV_SCORE_STEP(1) TKV_SCORE_STEP(2) TKV_SCORE_STEP(3) \
  }
      TKV_SCORE_GROUP(0)
      TKV_SCORE_GROUP(1)
      if constexpr (NG > 2) {
        TKV_SCORE_GROUP(2)
        TKV_SCORE_GROUP(3)
      }
    }
    // ---------------- mask, online softmax over the 8 scores of this lane
    float mx = -INFINITY;
    if ((live_a & live_b) == 0xFFFFu) {
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        sa[r4] *= a.scale_log2e;
        sb[r4] *= a.scale_log2e;
        mx = fmaxf(mx, fmaxf(sa[r4], sb[r4]));
      }
    } else {
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        sa[r4] = ((live_a >> (4 * qd + r4)) & 1u) ? sa[r4] * a.scale_log2e : -INFINITY;
        sb[r4] = ((live_b >> (4 * qd + r4)) & 1u) ? sb[r4] * a.scale_log2e : -INFINITY;
        mx = fmaxf(mx, fmaxf(sa[r4], sb[r4]));
      }
    }
    mx = col_max(mx);
    const float m_new = fmaxf(st.m, mx);
    const float m_safe = m_new == -INFINITY ? 0.f : m_new;
    if (__any(m_new != st.m)) {
      const float corr = __builtin_amdgcn_exp2f(st.m - m_safe);
#pragma unroll
      for (int mb = 0; mb < NM; ++mb) st.o[mb] *= corr;
#pragma unroll
      for (int g = 0; g < NG; ++g) st.ozp[g] *= corr;
      st.l *= corr;
      st.m = m_new;
    }
    float pa[4], pb[4];
#pragma unroll
    for (int r4 = 0; r4 < 4; ++r4) {
      pa[r4] = __builtin_amdgcn_exp2f(sa[r4] - m_safe);
      pb[r4] = __builtin_amdgcn_exp2f(sb[r4] - m_safe);
      st.l += pa[r4] + pb[r4];
    }
    // ---------------- values: per group, B = split(p * s_V), A = V codes; zero-point part on the VALU
#pragma unroll
    for (int g = 0; g < NG; ++g) {
      H8 pg;
#define TKV_P_STEP(R)                                                                                  \
  {                                                                                                    \
    constexpr int IA = (D == 128) ? (4 * R + GI) : (2 * R + GI);                                        \
    constexpr int IB = (D == 128) ? (4 * R + GI) : (8 + 2 * R + GI);                                    \
    xa[R] = pa[R] * bcast_row<IA>(vs_a);                                                               \
    xb[R] = pb[R] * bcast_row<IB>(D == 128 ? vs_b : vs_a);                                             \
    st.ozp[g] = fmaf(pa[R], bcast_row<IA>(vz_a), st.ozp[g]);                                           \
    st.ozp[g] = fmaf(pb[R], bcast_row<IB>(D == 128 ? vz_b : vz_a), st.ozp[g]);                         \
  }
#define TKV_P_GROUP(GI_)                \
  if (g == GI_) {                       \
    constexpr int GI = GI_;             \
    TKV_P_STEP(0) TKV_P_STEP(1) TKV_P_STEP(2) TKV_P_STEP(3) \
  }
      float xa[4], xb[4];
      TKV_P_GROUP(0)
      TKV_P_GROUP(1)
      if constexpr (NG > 2) {
        TKV_P_GROUP(2)
        TKV_P_GROUP(3)
      }
      // two-term split: high columns carry rne16(x), low columns rne16(x - rne16(x))
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        const uint32_t ha = pack_rne(xa[2 * i], xa[2 * i + 1]);
        const uint32_t hb = pack_rne(xb[2 * i], xb[2 * i + 1]);
        pg.u[i] = pack_rne(fmaf(-alpha, half_lo(ha), xa[2 * i]), fmaf(-alpha, half_hi(ha), xa[2 * i + 1]));
        pg.u[2 + i] = pack_rne(fmaf(-alpha, half_lo(hb), xb[2 * i]), fmaf(-alpha, half_hi(hb), xb[2 * i + 1]));
      }
#pragma unroll
      for (int mm = 0; mm < 2; ++mm) {
        const int mb = 2 * g + mm;
        H8 va;
        // k-slots 8qd+e: e<4 page a slots 4qd+e, e>=4 page b; field f = u*NM + mb holds slots (2u, 2u+1)
        va.u[0] = F::get(ra.vw, 0 * NM + mb);
        va.u[1] = F::get(ra.vw, 1 * NM + mb);
        va.u[2] = F::get(rb.vw, 0 * NM + mb);
        va.u[3] = F::get(rb.vw, 1 * NM + mb);
        st.o[mb] = __builtin_amdgcn_mfma_f32_16x16x32_f16(va.h, pg.h, st.o[mb], 0, 0, 0);
      }
    }
#undef TKV_SCORE_STEP
#undef TKV_SCORE_GROUP
#undef TKV_P_STEP
#undef TKV_P_GROUP
  }

  // Page ids and live masks of up to 64 pages are fetched with one vector load each (lane L
  // holds page p0 + base + L) and handed to the pair loop through v_readlane, so the loop
  // itself has no dependent scalar loads.  Occupancy, not software prefetch, hides the
  // latency of the packed-page loads: each wave has one page pair in flight.
  __device__ __forceinline__ void run() {
    const int n_pages = p1 - p0;
    for (int base = 0; base < n_pages; base += 64) {
      const int cnt = n_pages - base < 64 ? n_pages - base : 64;
      int vpid = 0;
      uint32_t vmask = 0;
      if (lane < cnt) {
        vpid = tab[p0 + base + lane];
        vmask = v.page_mask[cls][vpid] & 0xFFFFu;
      }
      if (a.window > 0) {
        // visibility of the 16 slots of each page: lane L walks the slots of its own page
        uint32_t vis = 0;
        if (lane < cnt) {
          const int32_t* sp = v.slot_pos[cls] + (int64_t)vpid * kPage;
#pragma unroll
          for (int t = 0; t < kPage; ++t) {
            const int d = qpos - sp[t];
            vis |= (d >= 0 && d < a.window) ? (1u << t) : 0u;
          }
        }
        vmask &= vis;
      }
      const int n_pairs = (cnt + 1) >> 1;
      for (int pr = wave; pr < n_pairs; pr += 4) {
        PairIds id;
        id.pid_a = __builtin_amdgcn_readlane(vpid, 2 * pr);
        id.live_a = __builtin_amdgcn_readlane(vmask, 2 * pr);
        const int ib = 2 * pr + 1 < cnt ? 2 * pr + 1 : 2 * pr;
        id.pid_b = __builtin_amdgcn_readlane(vpid, ib);
        id.live_b = 2 * pr + 1 < cnt ? __builtin_amdgcn_readlane(vmask, ib) : 0u;
        PairRegs<D, BITS> r;
        issue_loads(r, id);
        compute(r, id);
      }
    }
  }
};

template <int D, int G>
struct ItemLds {
  _Float16 q[G * D];
  float qsum[G * (D / 32)];
  float m[4][G], l[4][G];
  float acc[4][G][D];
};

// Everything one workgroup does for one item whose pages hold BITS-bit codes.
template <int D, int G, int BITS>
__device__ __forceinline__ void run_item(const thinkv_view& v, const DecodeArgs& a, ItemLds<D, G>& lds, int cls, int item, int ns,
                                         int np, int split, int hkv, int b, int seq) {
  constexpr int NG = D / 32, NM = D / 16;
  using F = Fld<BITS>;
  const thinkv_config& c = v.cfg;
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int Hq = c.n_q_heads;
  for (int i = tid; i < G * D; i += 256)
    lds.q[i] = (_Float16)load_as_f32(a.q, ((int64_t)b * Hq + hkv * G) * D + i, a.q_dtype);
  __syncthreads();
  if (tid < G * NG) {
    float s = 0.f;
    for (int i = 0; i < 32; ++i) s += (float)lds.q[(tid / NG) * D + 32 * (tid % NG) + i];
    lds.qsum[tid] = s;
  }
  __syncthreads();

  WaveState<D> st;
#pragma unroll
  for (int mb = 0; mb < NM; ++mb) st.o[mb] = float4v{0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int g = 0; g < NG; ++g) st.ozp[g] = 0.f;
  st.m = -INFINITY;
  st.l = 0.f;
  const int qpos = a.window > 0 ? a.q_pos[b] : 0;
  const int qd = lane >> 4, n = lane & 15;
  const int p0 = (int)((int64_t)item * np / ns), p1 = (int)((int64_t)(item + 1) * np / ns);
  const int32_t* tab = v.block_table + table_base(c, seq, a.layer, cls);
  {
    ClassRunner<D, BITS, G> cr(st, v, a, cls, tab, p0, p1, wave, hkv, lds.q, lds.qsum, qpos);
    cr.run();
  }

  // ---- fold: low-half columns into their heads, row groups for l and ozp, then the four waves
  float l = st.l;
  l += __shfl_xor(l, 16, 64);
  l += __shfl_xor(l, 32, 64);
  float ozp[NG];
#pragma unroll
  for (int g = 0; g < NG; ++g) {
    float z = st.ozp[g];
    z += __shfl_xor(z, 16, 64);
    z += __shfl_xor(z, 32, 64);
    ozp[g] = z;
  }
#pragma unroll
  for (int mb = 0; mb < NM; ++mb) {
    // V codes entered the MFMA as c * 2^(OMIN + rel(mb) - 24)
    const float unit = (float)(1 << (24 - F::OMIN - F::rel_of(mb)));
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      float x = st.o[mb][r];
      const float lo = __shfl(x, (lane & 48) | ((n + G) & 15), 64);
      x = (x + lo) * unit + ozp[mb >> 1];
      if (n < G) lds.acc[wave][n][16 * mb + 4 * qd + r] = x;
    }
  }
  if (qd == 0 && n < G) {
    lds.m[wave][n] = st.m;
    lds.l[wave][n] = l;
  }
  __syncthreads();
  for (int i = tid; i < G * D; i += 256) {
    const int g = i / D, ch = i % D;
    float M = -INFINITY;
#pragma unroll
    for (int w = 0; w < 4; ++w) M = fmaxf(M, lds.m[w][g]);
    float L = 0.f, A = 0.f;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const float f = (lds.m[w][g] == -INFINITY) ? 0.f : exp2f(lds.m[w][g] - M);
      L += lds.l[w][g] * f;
      A += lds.acc[w][g][ch] * f;
    }
    float* dst = a.partial + partial_index(a, Hq, D, b, hkv * G + g, split);
    dst[2 + ch] = A;
    if (ch == 0) {
      dst[0] = M;
      dst[1] = L;
    }
  }
}

template <int D, int G>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(3, 4))) void decode_mfma_kernel(thinkv_view v, DecodeArgs a) {
  const thinkv_config& c = v.cfg;
  const int split = blockIdx.x, hkv = blockIdx.y, b = blockIdx.z;
  const int seq = a.seq_ids[b];
  __shared__ ItemLds<D, G> lds;
  int np[3];
#pragma unroll
  for (int k = 0; k < 3; ++k) np[k] = (seq >= 0 && seq < c.max_seqs) ? v.n_pages[npages_index(c, seq, a.layer, k)] : 0;
  int cls, item, ns;
  if (!locate_item(a, np, split, &cls, &item, &ns)) return;
  const int bits = c.bits_of_class[cls];
  if (bits == 2)
    run_item<D, G, 2>(v, a, lds, cls, item, ns, np[cls], split, hkv, b, seq);
  else if (bits == 4)
    run_item<D, G, 4>(v, a, lds, cls, item, ns, np[cls], split, hkv, b, seq);
  else
    run_item<D, G, 8>(v, a, lds, cls, item, ns, np[cls], split, hkv, b, seq);
}

int decode_mfma_supported(const thinkv_config& c) {
  const int G = c.n_q_heads / c.n_kv_heads;
  return (c.head_dim == 64 || c.head_dim == 128) && G >= 1 && G <= 8;
}

template <int D>
static int launch_d(const thinkv_view& v, const DecodeArgs& a, hipStream_t st) {
  const int G = v.cfg.n_q_heads / v.cfg.n_kv_heads;
  dim3 grid(a.max_split, v.cfg.n_kv_heads, a.B), blk(256);
  switch (G) {
    case 1: hipLaunchKernelGGL((decode_mfma_kernel<D, 1>), grid, blk, 0, st, v, a); break;
    case 2: hipLaunchKernelGGL((decode_mfma_kernel<D, 2>), grid, blk, 0, st, v, a); break;
    case 3: hipLaunchKernelGGL((decode_mfma_kernel<D, 3>), grid, blk, 0, st, v, a); break;
    case 4: hipLaunchKernelGGL((decode_mfma_kernel<D, 4>), grid, blk, 0, st, v, a); break;
    case 5: hipLaunchKernelGGL((decode_mfma_kernel<D, 5>), grid, blk, 0, st, v, a); break;
    case 6: hipLaunchKernelGGL((decode_mfma_kernel<D, 6>), grid, blk, 0, st, v, a); break;
    case 7: hipLaunchKernelGGL((decode_mfma_kernel<D, 7>), grid, blk, 0, st, v, a); break;
    case 8: hipLaunchKernelGGL((decode_mfma_kernel<D, 8>), grid, blk, 0, st, v, a); break;
    default: return THINKV_E_SHAPE;
  }
  return hipGetLastError() == hipSuccess ? THINKV_OK : THINKV_E_HIP;
}

int launch_decode_mfma(const thinkv_view& v, const DecodeArgs& a, hipStream_t st) {
  return v.cfg.head_dim == 128 ? launch_d<128>(v, a, st) : launch_d<64>(v, a, st);
}

}  // namespace thinkv
