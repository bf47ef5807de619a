// The per-type runner of the decode kernel for the paper's number formats (THINKV_FMT_FP): FP8 E4M3 with a
// per-tensor scale, NVFP4 (E2M1 codes) and ternary codes with one E4M3 scale per 16 channels of the token.
//
// Same plan as for the integer formats (decode_mfma_kernel.h): the codes go to v_mfma_f32_16x16x32_f16 without being
// dequantised, the scales are applied to what the matrix cores return.  What differs:
//   * a code is a sign and a small IEEE-style magnitude.  An IEEE-style format nests in a wider one: the magnitude
//     bits placed right under a binary16 exponent ARE the code's value times a power of two (2^-14 for E2M1 and the
//     ternary bit, 2^-8 for E4M3), subnormal codes included; the sign goes to bit 15.  Two shifts and two masks per
//     operand register instead of the integer formats' one and a half;
//   * there are no zero-points, so the zero-point sums and the group sums of the query are gone;
//   * a group is 16 channels, half the K extent of the instruction: a slice of columns carries one group of 16, its
//     second operand is zero over the other half of the 32 channels, and there are twice as many column sets;
//   * an E4M3 scale is at most 448, so the lifted weights times the scale (times 2^-8: a scale byte shifted under a
//     binary16 exponent is the scale times 2^-8) always stay inside binary16: no check per pair;
//   * the 8-bit type has no scale per token: its tensor scales are folded into the exponent's factor (keys) and into
//     the tiles when the type is left (values).
#pragma once

namespace thinkv {

template <int BITS>
struct FldFp {
  static constexpr int FPH = 16 / BITS;
  static constexpr int EXP = BITS == 8 ? 8 : 14;   // operand = value of the code * 2^-EXP
  __device__ static __forceinline__ uint32_t shl(uint32_t x, int s) { return s >= 0 ? (x << s) : (x >> (-s)); }
  // operand register (two codes: low / high half) for field f of the chunk words w[]
  __device__ static __forceinline__ uint32_t get(const uint32_t* w, int f) {
    const int word = f / FPH, pos = f % FPH;
    const uint32_t x = w[word];
    if constexpr (BITS == 4) {          // [s e1 e0 m] at bits 4 pos .. 4 pos + 3 of each half
      return (shl(x, 9 - 4 * pos) & 0x0E000E00u) | ((x << (12 - 4 * pos)) & 0x80008000u);
    } else if constexpr (BITS == 2) {   // [s m] at bits 2 pos, 2 pos + 1
      return (shl(x, 10 - 2 * pos) & 0x04000400u) | ((x << (14 - 2 * pos)) & 0x80008000u);
    } else {                            // [s eeee mmm] in the low (pos 0) or high byte of each half
      if (pos == 0) return ((x & 0x007F007Fu) << 7) | ((x & 0x00800080u) << 8);
      return ((x >> 1) & 0x3F803F80u) | (x & 0x80008000u);
    }
  }
};

template <int D, int GP>
struct ColsFp {
  static constexpr int NG = D / 16;                           // groups of 16 channels
  static constexpr int CS = (16 / GP) < NG ? (16 / GP) : NG;   // groups (slices) per column set: 2 or 4
  static constexpr int NSET = NG / CS;
};

template <int D, int BITS, int NSET>
struct PageRegsFp {
  static constexpr int CW = (D / 32) * BITS / 4;
  uint32_t kw[CW], vw[CW];
  uint32_t km[NSET], vm[NSET];   // the E4M3 scale bytes of (the slice's group, the lane's four slots); unused at 8 bits
};
template <int D, int BITS, int NSET>
struct PairRegsFp {
  PageRegsFp<D, BITS, NSET> a, b;
};

// per column set the eight binary16 values of (the lane's head, channels 32 G + 8 qd ..) where those channels lie in
// the group of 16 of the lane's slice; zeros otherwise
template <int NSET>
struct QRegsFp {
  H8 q[NSET];
};

// four scale bytes (slots 0..3 of the lane's quad) -> two registers of binary16 pairs, each scale times 2^-8
__device__ __forceinline__ void scales_to_halves(uint32_t bytes, uint32_t& lo, uint32_t& hi) {
  lo = __builtin_amdgcn_perm(0u, bytes, 0x0C010C00u) << 7;
  hi = __builtin_amdgcn_perm(0u, bytes, 0x0C030C02u) << 7;
}

// STAT: besides attending, leave the group-pooled score of every visited slot for the attention-sparsity statistic
// (as the integer-format runner does).
template <int D, int BITS, int GP, bool STAT>
struct ClassRunnerFp : PairWalk<ClassRunnerFp<D, BITS, GP, STAT>, PairRegsFp<D, BITS, ColsFp<D, GP>::NSET>> {
  using CL = ColsFp<D, GP>;
  static constexpr int NG32 = D / 32, NM = D / 16, CS = CL::CS, NSET = CL::NSET;
  static constexpr bool kHalfPipe = false;
  static constexpr int kLift = 14;   // 2^14 * 448 * 2^-8 < 65504: the lifted second operand of the value products cannot overflow
  using F = FldFp<BITS>;
  using Pair = PairRegsFp<D, BITS, NSET>;
  using Walk = PairWalk<ClassRunnerFp<D, BITS, GP, STAT>, Pair>;
  using Walk::v;
  using Walk::a;
  using Walk::cls;
  using Walk::hkv;
  using Walk::lane;
  WaveState<D, NSET>& st;
  int qd, n;
  int meta_off[NSET];   // byte offset, inside a meta region, of the lane's four scale bytes per column set
  H8 bq[NG32];          // B operands of the score MFMAs: q over the half of the 32 channels that is the slice's group, zeros elsewhere
  float kappa;          // MFMA score units -> log2 domain
  float tile_out;       // tiles -> absolute units / 2^24 when the type is left
  float neg1;
  float* stat;          // STAT: pooled scores of this type's page list, 16 per page
  int stat_room;        // STAT: pages of this list the buffer has room for
  bool head_ok;         // this lane's column belongs to a query head of the group

  __device__ __forceinline__ ClassRunnerFp(WaveState<D, NSET>& st_, const thinkv_view& v_, const DecodeArgs& a_, int cls_, const int32_t* tab_,
                                           int p0_, int p1_, int hkv_, int G, const QRegsFp<NSET>& qr, int qpos_, float* stat_, int stat_room_)
      : Walk(v_, a_, cls_, hkv_, qpos_, tab_, p0_, p1_), st(st_), stat(stat_), stat_room(stat_room_) {
    qd = lane >> 4;
    n = lane & 15;
    const int gl = n / GP;
    head_ok = n % GP < G;
    const int glc = gl < CS ? gl : CS - 1;
    neg1 = -1.0f;
    asm volatile("" : "+v"(neg1));
    const thinkv_config& c = v.cfg;
    if constexpr (BITS == 8) {
      kappa = 256.0f * c.fp8_scale[0] * a.scale_log2e;
      tile_out = c.fp8_scale[1] * (1.0f / (float)(1 << 16)) * (1.0f / (float)(1 << kLift));
    } else {
      kappa = 4194304.0f * a.scale_log2e;                                   // 2^14 (codes) * 2^8 (scales)
      tile_out = 0.25f * (1.0f / (float)(1 << kLift));                      // 2^(14 + 8 - 24 - lift)
    }
#pragma unroll
    for (int s = 0; s < NSET; ++s) meta_off[s] = (s * CS + glc) * kPage + 4 * qd;
#pragma unroll
    for (int g = 0; g < NG32; ++g) {
      const int set = (2 * g) / CS;
      const bool on = gl < CS && ((set * CS + gl) >> 1) == g;
#pragma unroll
      for (int w = 0; w < 4; ++w) bq[g].u[w] = on ? qr.q[set].u[w] : 0u;
    }
    // enter the type: the denominator and the tiles take the lift, the tiles the units of the type
    st.l *= (float)(1 << kLift);
    const float in = 1.0f / tile_out;
#pragma unroll
    for (int mb = 0; mb < NM; ++mb) st.o[mb] *= in;
  }
  __device__ __forceinline__ void leave() {
    st.l *= 1.0f / (float)(1 << kLift);
#pragma unroll
    for (int mb = 0; mb < NM; ++mb) st.o[mb] *= tile_out;
  }

  __device__ __forceinline__ void issue_loads(Pair& r, const PairIds& id) const {
    constexpr int CW = PageRegsFp<D, BITS, NSET>::CW;
    const int H = v.cfg.n_kv_heads;
    const BlockGeom g = block_geom(BITS, D, THINKV_FMT_FP);
    const uint8_t* blk[2] = {v.arena[cls] + ((int64_t)id.pid_a * H + hkv) * g.block_bytes, v.arena[cls] + ((int64_t)id.pid_b * H + hkv) * g.block_bytes};
#pragma unroll
    for (int pg = 0; pg < 2; ++pg) {
      PageRegsFp<D, BITS, NSET>& x = pg ? r.b : r.a;
      const uint32_t* kc = (const uint32_t*)(blk[pg] + g.k_codes) + lane * CW;
      const uint32_t* vc = (const uint32_t*)(blk[pg] + g.v_codes) + lane * CW;
      if constexpr (CW == 1) {
        x.kw[0] = kc[0];
        x.vw[0] = vc[0];
      } else if constexpr (CW == 2) {
        const uint2 p = ld8<true>(kc), q = ld8<true>(vc);
        x.kw[0] = p.x; x.kw[1] = p.y;
        x.vw[0] = q.x; x.vw[1] = q.y;
      } else {
#pragma unroll
        for (int i = 0; i < CW; i += 4) {
          const uint4 p = ld16<true>(kc + i), q = ld16<true>(vc + i);
          x.kw[i] = p.x; x.kw[i + 1] = p.y; x.kw[i + 2] = p.z; x.kw[i + 3] = p.w;
          x.vw[i] = q.x; x.vw[i + 1] = q.y; x.vw[i + 2] = q.z; x.vw[i + 3] = q.w;
        }
      }
      if constexpr (BITS != 8) {
#pragma unroll
        for (int s = 0; s < NSET; ++s) {
          x.km[s] = *(const uint32_t*)(blk[pg] + g.k_meta + meta_off[s]);
          x.vm[s] = *(const uint32_t*)(blk[pg] + g.v_meta + meta_off[s]);
        }
      }
    }
  }

  // scores of one page for this lane's four tokens, in MFMA units (times kappa = log2 domain)
  __device__ __forceinline__ void page_scores(const PageRegsFp<D, BITS, NSET>& r, float* s) const {
    const float4v zero = {0.f, 0.f, 0.f, 0.f};
    float4v c[NSET];
#pragma unroll
    for (int g = 0; g < NG32; ++g) {
      const int set = (2 * g) / CS;
      const bool first = (2 * g) % CS == 0;
      H8 ka;
#pragma unroll
      for (int vv = 0; vv < 4; ++vv) ka.u[vv] = F::get(r.kw, 4 * g + vv);
      c[set] = __builtin_amdgcn_mfma_f32_16x16x32_f16(ka.h, bq[g].h, first ? zero : c[set], 0, 0, 0);
    }
    float acc[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int set = 0; set < NSET; ++set) {
      if constexpr (BITS == 8) {
#pragma unroll
        for (int R = 0; R < 4; ++R) acc[R] = set == 0 ? c[set][R] : acc[R] + c[set][R];
      } else {
        uint32_t lo, hi;
        scales_to_halves(r.km[set], lo, hi);
        acc[0] = fmaf(half_lo(lo), c[set][0], acc[0]);
        acc[1] = fmaf(half_hi(lo), c[set][1], acc[1]);
        acc[2] = fmaf(half_lo(hi), c[set][2], acc[2]);
        acc[3] = fmaf(half_hi(hi), c[set][3], acc[3]);
      }
    }
#pragma unroll
    for (int R = 0; R < 4; ++R) {
      float t = add_row_ror<8>(acc[R]);
      if constexpr (GP == 4) t = add_row_ror<4>(t);
      s[R] = t;
    }
  }

  __device__ __forceinline__ void compute(const Pair& r, const PairIds& id) {
    const uint32_t live_a = id.live_a, live_b = id.live_b;
    float sa[4], sb[4];
    page_scores(r.a, sa);
    page_scores(r.b, sb);
    if ((live_a & live_b) != 0xFFFFu) {   // dead slots: score -inf, hence p = 0 (their stale codes and scales are finite)
      const uint32_t la = (live_a >> (4 * qd)) & 0xFu, lb = (live_b >> (4 * qd)) & 0xFu;
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        sa[r4] = ((la >> r4) & 1u) ? sa[r4] : -INFINITY;
        sb[r4] = ((lb >> r4) & 1u) ? sb[r4] : -INFINITY;
      }
    }
    if constexpr (STAT) {
      // pooled scores: maximum over the heads of the group, i.e. over the GP lanes of a slice (all slices hold the
      // same totals); the lanes of column 0 store their four slots of each page
      auto pooled = [&](const float* sc, int idx) {
        float u[4];
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
          u[r4] = head_ok ? sc[r4] * kappa : -INFINITY;
          u[r4] = max_dpp<0x4E>(max_dpp<0xB1>(u[r4]));
          if constexpr (GP == 8) u[r4] = max_dpp<0x124>(u[r4]);
        }
        if (n == 0 && idx >= 0 && idx < stat_room) *(float4*)(stat + (int64_t)idx * kPage + 4 * qd) = make_float4(u[0], u[1], u[2], u[3]);
      };
      pooled(sa, id.idx_a);
      pooled(sb, id.idx_b);
    }
    const float mx = fmaxf(fmaxf(fmaxf(sa[0], sa[1]), fmaxf(sa[2], sa[3])), fmaxf(fmaxf(sb[0], sb[1]), fmaxf(sb[2], sb[3]))) * kappa;
    if (__any(mx > st.m)) {
      const float m_new = fmaxf(st.m, col_max(mx));
      const float m_sub = m_new == -INFINITY ? 0.f : m_new;
      const float corr = __builtin_amdgcn_exp2f(st.m - m_sub);
#pragma unroll
      for (int mb = 0; mb < NM; ++mb) st.o[mb] *= corr;
      st.l *= corr;
      st.m = m_new;
      st.m_sub = m_sub;
    }
    float pa[4], pb[4];
    const float mref = st.m_sub - (float)kLift;
#pragma unroll
    for (int r4 = 0; r4 < 4; ++r4) {
      pa[r4] = __builtin_amdgcn_exp2f(fmaf(sa[r4], kappa, -mref));
      pb[r4] = __builtin_amdgcn_exp2f(fmaf(sb[r4], kappa, -mref));
    }
    st.l += ((pa[0] + pa[1]) + (pa[2] + pa[3])) + ((pb[0] + pb[1]) + (pb[2] + pb[3]));
    // values, per column set: B = two-term split of p * s_V, A = V codes
    H8 hi, lo;
#pragma unroll
    for (int set = 0; set < NSET; ++set) {
      if (BITS != 8 || set == 0) {
        float xa[4], xb[4];
        if constexpr (BITS == 8) {
#pragma unroll
          for (int r4 = 0; r4 < 4; ++r4) {
            xa[r4] = pa[r4];
            xb[r4] = pb[r4];
          }
        } else {
          uint32_t al, ah, bl, bh;
          scales_to_halves(r.a.vm[set], al, ah);
          scales_to_halves(r.b.vm[set], bl, bh);
          xa[0] = fmaf(half_lo(al), pa[0], 0.0f); xa[1] = fmaf(half_hi(al), pa[1], 0.0f);
          xa[2] = fmaf(half_lo(ah), pa[2], 0.0f); xa[3] = fmaf(half_hi(ah), pa[3], 0.0f);
          xb[0] = fmaf(half_lo(bl), pb[0], 0.0f); xb[1] = fmaf(half_hi(bl), pb[1], 0.0f);
          xb[2] = fmaf(half_lo(bh), pb[2], 0.0f); xb[3] = fmaf(half_hi(bh), pb[3], 0.0f);
        }
        // k-slots 8qd+e: e<4 page a slots 4qd+e, e>=4 page b
        hi.u[0] = pack_rne(xa[0], xa[1]);
        hi.u[1] = pack_rne(xa[2], xa[3]);
        hi.u[2] = pack_rne(xb[0], xb[1]);
        hi.u[3] = pack_rne(xb[2], xb[3]);
        lo.u[0] = pack_rne(fmaf(neg1, half_lo(hi.u[0]), xa[0]), fmaf(neg1, half_hi(hi.u[0]), xa[1]));
        lo.u[1] = pack_rne(fmaf(neg1, half_lo(hi.u[1]), xa[2]), fmaf(neg1, half_hi(hi.u[1]), xa[3]));
        lo.u[2] = pack_rne(fmaf(neg1, half_lo(hi.u[2]), xb[0]), fmaf(neg1, half_hi(hi.u[2]), xb[1]));
        lo.u[3] = pack_rne(fmaf(neg1, half_lo(hi.u[3]), xb[2]), fmaf(neg1, half_hi(hi.u[3]), xb[3]));
      }
#pragma unroll
      for (int mm = 0; mm < CS; ++mm) {
        const int mb = CS * set + mm;   // a 16-channel block is a group
        H8 va;
        va.u[0] = F::get(r.a.vw, 0 * NM + mb);
        va.u[1] = F::get(r.a.vw, 1 * NM + mb);
        va.u[2] = F::get(r.b.vw, 0 * NM + mb);
        va.u[3] = F::get(r.b.vw, 1 * NM + mb);
        st.o[mb] = __builtin_amdgcn_mfma_f32_16x16x32_f16(va.h, hi.h, st.o[mb], 0, 0, 0);
        st.o[mb] = __builtin_amdgcn_mfma_f32_16x16x32_f16(va.h, lo.h, st.o[mb], 0, 0, 0);
      }
    }
  }
};

}  // namespace thinkv
