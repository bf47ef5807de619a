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
// scales multiply whole MFMA results in binary32; the zero-point terms are two small MFMAs of
// their own (stored binary16 zero-points against a two-term split of the group sums of q, and
// against a two-term split of p, which also yields the softmax denominator from a row of ones).
// Scores are computed transposed (tokens x heads) so that their register layout is already
// the B-operand layout of the PV product; the 16 MFMA columns carry the G query heads of the
// group, a duplicate of them that takes the low half of the two-term binary16 splits
// (22 significant bits), and padding.  Per-token scales reach the lanes that need them
// through DPP row broadcasts.
//
// One workgroup of four waves per (query, kv-head, item); an item holds an equal share of the
// pages of every thought type and walks them type by type, so the bit width is a
// compile-time constant of each inner loop; a wave takes every fourth page pair; the four
// waves are merged through LDS into one partial (m, l, acc) per query head.
#include "decode_common.h"

namespace thinkv {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half4 __attribute__((ext_vector_type(4)));
typedef _Float16 half2v __attribute__((ext_vector_type(2)));
typedef float float4v __attribute__((ext_vector_type(4)));
typedef float float2v __attribute__((ext_vector_type(2)));

union H8 {
  half8 h;
  uint32_t u[4];
};
union H4 {
  half4 h;
  uint32_t u[2];
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

// two-term binary16 split of (x0, x1): returns rne16(x) in "high" lanes (alpha = 0) and
// rne16(x - rne16(x)) in "low" lanes (alpha = 1); high + low carries 22 significant bits.
__device__ __forceinline__ uint32_t split2(float x0, float x1, float alpha) {
  const uint32_t h = pack_rne(x0, x1);
  return pack_rne(fmaf(-alpha, half_lo(h), x0), fmaf(-alpha, half_hi(h), x1));
}

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

// What one lane holds of one page: its K and V chunks, one K scale and one V scale (to be
// broadcast along its row of 16 lanes), the K zero-points of its slot (A operand of the
// score zero-point MFMA) and the V zero-points of four slots of its group (A operand of the
// output zero-point MFMA).
template <int D, int BITS>
struct PageRegs {
  static constexpr int CW = (D / 32) * BITS / 4;  // chunk dwords
  static constexpr int ZW = D / 64;               // dwords of K zero-points per slot
  uint32_t kw[CW], vw[CW];
  uint32_t kzp[ZW], vzp[2];
  uint16_t ks, vs;
};

template <int D, int BITS>
__device__ __forceinline__ void load_page(PageRegs<D, BITS>& r, const uint8_t* blk, int lane, int scale_idx) {
  constexpr int CW = PageRegs<D, BITS>::CW, NG = D / 32;
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
  r.ks = ((const uint16_t*)(blk + g.k_scale))[scale_idx];
  r.vs = ((const uint16_t*)(blk + g.v_scale))[scale_idx];
  const int t = lane & 15, qd = lane >> 4;
  if constexpr (D == 128) {
    const uint2 z = ((const uint2*)(blk + g.k_zp))[t];        // slot t, groups 0..3
    r.kzp[0] = z.x; r.kzp[1] = z.y;
  } else {
    r.kzp[0] = ((const uint32_t*)(blk + g.k_zp))[t];          // slot t, groups 0..1
  }
  const uint2 z = *(const uint2*)(blk + g.v_zp + ((t & (NG - 1)) * kPage + 4 * qd) * 2);   // group t%NG, slots 4qd..4qd+3
  r.vzp[0] = z.x; r.vzp[1] = z.y;
}

template <int D>
struct WaveState {
  static constexpr int NG = D / 32, NM = D / 16;
  float4v o[NM];   // o[mb][r]: channel 16*mb + 4*qd + r of column n, in units of the class
  float4v oz;      // rows 0..NG-1: zero-point part of the output per group; row NG: sum of p
  float m;         // running maximum (log2 domain) of column n
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

// One wave's share of an item: page pairs wave, wave+4, ... of tab[p0..p1).
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
  H8 bq[NG];          // B operand of the score MFMAs
  H4 bqs;             // B operand of the score zero-point MFMA: split of scale * sum_{i in g} q_i
  uint32_t zmask, zones;  // A-operand row selection of the output zero-point MFMA
  float kscale;       // 2^(24 - OMIN) * softmax_scale * log2(e)

  __device__ __forceinline__ ClassRunner(WaveState<D>& st_, const thinkv_view& v_, const DecodeArgs& a_, int cls_, const int32_t* tab_,
                                         int p0_, int p1_, int wave_, int hkv_, const _Float16* s_q, const float* s_qsum, int qpos_)
      : st(st_), v(v_), a(a_), cls(cls_), hkv(hkv_), qpos(qpos_), tab(tab_), p0(p0_), p1(p1_), wave(wave_) {
    lane = threadIdx.x & 63;
    qd = lane >> 4;
    n = lane & 15;
    alpha = (n >= G && n < 2 * G) ? 1.0f : 0.0f;
    kscale = (float)(1 << (24 - F::OMIN)) * a.scale_log2e;
    const bool used = n < 2 * G;
    const int head = n < G ? n : n - G;
    // q of column n, channels (g, 8qd+e), scaled down by the residual power of two its code carries
#pragma unroll
    for (int g = 0; g < NG; ++g) {
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const int f = 4 * g + (e >> 1);
        float x = used ? (float)s_q[head * D + 32 * g + 8 * qd + e] : 0.f;
        x *= 1.0f / (float)(1 << F::rel_of(f));
        bq[g].h[e] = (_Float16)x;   // exact: power-of-two scaling of a binary16 value
      }
    }
    // k-slots of the 16x16x16 zero-point MFMA: D=128: (g0..g3) high terms in k 0..3 (row
    // group 0), low terms in k 4..7 (row group 1); D=64: (g0, g1, g0, g1) = high, high, low, low
    float qs[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int g = i % NG;
      const float x = used ? s_qsum[head * NG + g] * a.scale_log2e : 0.f;
      const float hi = (float)(_Float16)x;
      const bool low_term = NG == 4 ? (qd == 1) : (i >= 2);
      const bool live = NG == 4 ? (qd < 2) : (qd == 0);
      qs[i] = live ? (low_term ? x - hi : hi) : 0.f;
    }
    bqs.u[0] = pack_rne(qs[0], qs[1]);
    bqs.u[1] = pack_rne(qs[2], qs[3]);
    // rows of the output zero-point MFMA: m < NG -> zero-points of group m, m == NG -> ones
    zmask = n < NG ? 0xFFFFFFFFu : 0u;
    zones = n == NG ? 0x3C003C00u : 0u;
  }

  __device__ __forceinline__ void issue_loads(PairRegs<D, BITS>& r, const PairIds& id) const {
    const int H = v.cfg.n_kv_heads;
    const BlockGeom geo = block_geom(BITS, D);
    const uint8_t* blk_a = v.arena[cls] + ((int64_t)id.pid_a * H + hkv) * geo.block_bytes;
    const uint8_t* blk_b = v.arena[cls] + ((int64_t)id.pid_b * H + hkv) * geo.block_bytes;
    if constexpr (D == 128) {
      load_page<D, BITS>(r.a, blk_a, lane, lane);            // scale of (slot lane/4, group lane%4)
      load_page<D, BITS>(r.b, blk_b, lane, lane);
    } else {
      // 32 scales per page: lanes x<8 of every row take page a, x>=8 page b
      const int si = 8 * qd + (n & 7);
      load_page<D, BITS>(r.a, blk_a, lane, si);
      load_page<D, BITS>(r.b, blk_b, lane, si);
    }
  }

  __device__ __forceinline__ void compute(const PairRegs<D, BITS>& r, const PairIds& id) {
    const uint32_t live_a = id.live_a, live_b = id.live_b;
    const PageRegs<D, BITS>& ra = r.a;
    const PageRegs<D, BITS>& rb = r.b;
    // scales to broadcast: D=128 one register per page; D=64 both pages share a register
    uint16_t ksa = ra.ks, vsa = ra.vs;
    if constexpr (D == 64) {
      if (n >= 8) { ksa = rb.ks; vsa = rb.vs; }
    }
    const float ks_a = (float)__builtin_bit_cast(_Float16, ksa) * kscale;
    const float vs_a = (float)__builtin_bit_cast(_Float16, vsa);
    float ks_b = ks_a, vs_b = vs_a;
    if constexpr (D == 128) {
      ks_b = (float)__builtin_bit_cast(_Float16, rb.ks) * kscale;
      vs_b = (float)__builtin_bit_cast(_Float16, rb.vs);
    }

    // ---------------- scores: S^T[token][column] per page, log2 domain
    // zero-point term first: zp_K[token][g] x split(scale * qsum[g][column])
    H4 za, zb;
    if constexpr (D == 128) {
      za.u[0] = ra.kzp[0]; za.u[1] = ra.kzp[1];
      zb.u[0] = rb.kzp[0]; zb.u[1] = rb.kzp[1];
    } else {
      za.u[0] = za.u[1] = ra.kzp[0];
      zb.u[0] = zb.u[1] = rb.kzp[0];
    }
    const float4v zero = {0.f, 0.f, 0.f, 0.f};
    float4v sa = __builtin_amdgcn_mfma_f32_16x16x16f16(za.h, bqs.h, zero, 0, 0, 0);
    float4v sb = __builtin_amdgcn_mfma_f32_16x16x16f16(zb.h, bqs.h, zero, 0, 0, 0);
#pragma unroll
    for (int g = 0; g < NG; ++g) {
      H8 ka, kb;
#pragma unroll
      for (int vv = 0; vv < 4; ++vv) {
        ka.u[vv] = F::get(ra.kw, 4 * g + vv);
        kb.u[vv] = F::get(rb.kw, 4 * g + vv);
      }
      const float4v ya = __builtin_amdgcn_mfma_f32_16x16x32_f16(ka.h, bq[g].h, zero, 0, 0, 0);
      const float4v yb = __builtin_amdgcn_mfma_f32_16x16x32_f16(kb.h, bq[g].h, zero, 0, 0, 0);
      // the scale of (token 4qd+r, group g) sits in lane 4r+g of this row (D=128),
      // or lane 8p+2r+g (D=64, p = page)
#define TKV_SCORE_STEP(R)                                                                              \
  {                                                                                                    \
    constexpr int IA = (D == 128) ? (4 * R + GI) : (2 * R + GI);                                        \
    constexpr int IB = (D == 128) ? (4 * R + GI) : (8 + 2 * R + GI);                                    \
    sa[R] = fmaf(bcast_row<IA>(ks_a), ya[R], sa[R]);                                                   \
    sb[R] = fmaf(bcast_row<IB>(D == 128 ? ks_b : ks_a), yb[R], sb[R]);                                 \
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
    if ((live_a & live_b) != 0xFFFFu) {
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        sa[r4] = ((live_a >> (4 * qd + r4)) & 1u) ? sa[r4] : -INFINITY;
        sb[r4] = ((live_b >> (4 * qd + r4)) & 1u) ? sb[r4] : -INFINITY;
      }
    }
    float mx = fmaxf(fmaxf(fmaxf(sa[0], sa[1]), fmaxf(sa[2], sa[3])), fmaxf(fmaxf(sb[0], sb[1]), fmaxf(sb[2], sb[3])));
    mx = col_max(mx);
    const float m_new = fmaxf(st.m, mx);
    const float m_safe = m_new == -INFINITY ? 0.f : m_new;
    if (__any(m_new != st.m)) {
      const float corr = __builtin_amdgcn_exp2f(st.m - m_safe);
#pragma unroll
      for (int mb = 0; mb < NM; ++mb) st.o[mb] *= corr;
      st.oz *= corr;
      st.m = m_new;
    }
    float pa[4], pb[4];
#pragma unroll
    for (int r4 = 0; r4 < 4; ++r4) {
      pa[r4] = __builtin_amdgcn_exp2f(sa[r4] - m_safe);
      pb[r4] = __builtin_amdgcn_exp2f(sb[r4] - m_safe);
    }
    // ---------------- zero-point part of the output and the softmax denominator:
    // rows = (zp_V of group 0..NG-1, ones) x split(p)
    {
      H8 zp, pz;
      zp.u[0] = (ra.vzp[0] & zmask) | zones;
      zp.u[1] = (ra.vzp[1] & zmask) | zones;
      zp.u[2] = (rb.vzp[0] & zmask) | zones;
      zp.u[3] = (rb.vzp[1] & zmask) | zones;
      pz.u[0] = split2(pa[0], pa[1], alpha);
      pz.u[1] = split2(pa[2], pa[3], alpha);
      pz.u[2] = split2(pb[0], pb[1], alpha);
      pz.u[3] = split2(pb[2], pb[3], alpha);
      st.oz = __builtin_amdgcn_mfma_f32_16x16x32_f16(zp.h, pz.h, st.oz, 0, 0, 0);
    }
    // ---------------- values: per group, B = split(p * s_V), A = V codes
#pragma unroll
    for (int g = 0; g < NG; ++g) {
      H8 pg;
      float xa[4], xb[4];
#define TKV_P_STEP(R)                                                                                  \
  {                                                                                                    \
    constexpr int IA = (D == 128) ? (4 * R + GI) : (2 * R + GI);                                        \
    constexpr int IB = (D == 128) ? (4 * R + GI) : (8 + 2 * R + GI);                                    \
    xa[R] = pa[R] * bcast_row<IA>(vs_a);                                                               \
    xb[R] = pb[R] * bcast_row<IB>(D == 128 ? vs_b : vs_a);                                             \
  }
#define TKV_P_GROUP(GI_)                \
  if (g == GI_) {                       \
    constexpr int GI = GI_;             \
    TKV_P_STEP(0) TKV_P_STEP(1) TKV_P_STEP(2) TKV_P_STEP(3) \
  }
      TKV_P_GROUP(0)
      TKV_P_GROUP(1)
      if constexpr (NG > 2) {
        TKV_P_GROUP(2)
        TKV_P_GROUP(3)
      }
      pg.u[0] = split2(xa[0], xa[1], alpha);
      pg.u[1] = split2(xa[2], xa[3], alpha);
      pg.u[2] = split2(xb[0], xb[1], alpha);
      pg.u[3] = split2(xb[2], xb[3], alpha);
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
        if ((id.live_a | id.live_b) == 0) continue;
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

template <int D>
__device__ __forceinline__ float class_unit(int bits, int mb) {
  // V codes of a b-bit class enter the MFMA as c * 2^(OMIN + rel(mb) - 24)
  const int sh = bits == 2 ? Fld<2>::OMIN + Fld<2>::rel_of(mb) : (bits == 4 ? Fld<4>::OMIN + Fld<4>::rel_of(mb) : 0);
  return (float)(1 << sh);
}

// One workgroup of four waves per (query, kv-head, item).
template <int D, int G>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(3, 4))) void decode_mfma_kernel(thinkv_view v, DecodeArgs a) {
  constexpr int NG = D / 32, NM = D / 16;
  const thinkv_config& c = v.cfg;
  const int split = blockIdx.x, hkv = blockIdx.y, b = blockIdx.z;
  const int seq = a.seq_ids[b];
  __shared__ ItemLds<D, G> lds;
  int np[3], np_total = 0;
#pragma unroll
  for (int k = 0; k < 3; ++k) {
    np[k] = (seq >= 0 && seq < c.max_seqs) ? v.n_pages[npages_index(c, seq, a.layer, k)] : 0;
    np_total += np[k];
  }
  const int ns = n_items_of(a, np_total);
  if (split >= ns) return;

  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int Hq = c.n_q_heads;
  for (int i = tid; i < G * D; i += 256)
    lds.q[i] = (_Float16)load_as_f32(a.q, ((int64_t)b * Hq + hkv * G) * D + i, a.q_dtype);
  __syncthreads();
  if (tid < G * NG * 4) {
    // four threads per (head, group) sum eight channels each
    const int hg = tid >> 2, part = tid & 3;
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) s += (float)lds.q[(hg / NG) * D + 32 * (hg % NG) + 8 * part + i];
    s += __shfl_xor(s, 1, 64);
    s += __shfl_xor(s, 2, 64);
    if (part == 0) lds.qsum[hg] = s;
  }
  __syncthreads();

  WaveState<D> st;
#pragma unroll
  for (int mb = 0; mb < NM; ++mb) st.o[mb] = float4v{0.f, 0.f, 0.f, 0.f};
  st.oz = float4v{0.f, 0.f, 0.f, 0.f};
  st.m = -INFINITY;
  const int qpos = a.window > 0 ? a.q_pos[b] : 0;
  const int qd = lane >> 4, n = lane & 15;

  // The running output is kept in the units of the class being walked (its codes carry a
  // power of two that depends on the bit width) and re-based at class boundaries.
  for (int k = 0; k < 3; ++k) {
    const int bits = c.bits_of_class[k];
    const int p0 = (int)((int64_t)split * np[k] / ns), p1 = (int)((int64_t)(split + 1) * np[k] / ns);
    if (p1 <= p0) continue;
    const int32_t* tab = v.block_table + table_base(c, seq, a.layer, k);
#pragma unroll
    for (int mb = 0; mb < NM; ++mb) st.o[mb] *= class_unit<D>(bits, mb);
    if (bits == 2) {
      ClassRunner<D, 2, G> cr(st, v, a, k, tab, p0, p1, wave, hkv, lds.q, lds.qsum, qpos);
      cr.run();
    } else if (bits == 4) {
      ClassRunner<D, 4, G> cr(st, v, a, k, tab, p0, p1, wave, hkv, lds.q, lds.qsum, qpos);
      cr.run();
    } else {
      ClassRunner<D, 8, G> cr(st, v, a, k, tab, p0, p1, wave, hkv, lds.q, lds.qsum, qpos);
      cr.run();
    }
#pragma unroll
    for (int mb = 0; mb < NM; ++mb) st.o[mb] *= 1.0f / class_unit<D>(bits, mb);
  }

  // ---- fold.  The zero-point MFMA left rows 0..NG-1 = zero-point part of the output per
  // group and row NG = sum of p (rows 0..3 live in row group 0, row 4 in row group 1);
  // high and low columns are added, then every lane of the column fetches what it needs.
  float zsum[NG], l;
  {
    float t[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) t[r] = st.oz[r] + __shfl(st.oz[r], (lane & 48) | ((n + G) & 15), 64);
#pragma unroll
    for (int g = 0; g < NG; ++g) zsum[g] = __shfl(t[g], n, 64);
    l = NG == 4 ? __shfl(t[0], 16 + n, 64) : __shfl(t[2], n, 64);
  }
#pragma unroll
  for (int mb = 0; mb < NM; ++mb) {
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      float x = st.o[mb][r];
      const float lo = __shfl(x, (lane & 48) | ((n + G) & 15), 64);
      x = (x + lo) * 16777216.f + zsum[mb >> 1];
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
