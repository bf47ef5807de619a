// Shared device/host helpers for the ThinKV kernels (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/thinkv.h"

namespace thinkv {

constexpr int kPage = THINKV_PAGE_SIZE;   // slots per page
constexpr int kGroup = THINKV_GROUP_SIZE; // channels per quantisation group
constexpr int kWave = 64;

// Geometry of one (page, kv-head) block for b-bit codes and head_dim D.
// [K codes][K meta][V codes][V meta]; a meta region is NG*4 units of 16 bytes, unit
// (group g, slot quad qd) = g*4 + qd holding eight binary16: the scales of slots
// 4qd..4qd+3 of group g, then their zero-points.
struct BlockGeom {
  int chunk_bytes;  // CB = (D/32)*b
  int codes_bytes;  // 64*CB
  int meta_bytes;   // 16*(D/32)*4: scales and zero-points of one of K / V
  int k_codes, k_meta, v_codes, v_meta;  // region offsets
  int block_bytes;
};

// fmt THINKV_FMT_FP: the code regions are the same; a meta region is one E4M3 scale byte per (slot, group
// of 16 channels), byte group16 * 16 + slot, and there is none for the 8-bit type (per-tensor scale).
constexpr int kGroupFp = 16;
__host__ __device__ inline BlockGeom block_geom(int bits, int D, int fmt = THINKV_FMT_INT) {
  BlockGeom g;
  g.chunk_bytes = (D / kGroup) * bits;
  g.codes_bytes = 64 * g.chunk_bytes;
  g.meta_bytes = fmt == THINKV_FMT_FP ? (bits == 8 ? 0 : kPage * (D / kGroupFp)) : kPage * (D / kGroup) * 4;
  g.k_codes = 0;
  g.k_meta = g.codes_bytes;
  g.v_codes = g.k_meta + g.meta_bytes;
  g.v_meta = g.v_codes + g.codes_bytes;
  g.block_bytes = 2 * (g.codes_bytes + g.meta_bytes);
  return g;
}

// index (in binary16 units) of the scale of (slot t, group g) inside a meta region; its
// zero-point sits four places further
__host__ __device__ inline int meta_index(int t, int g) { return (g * 4 + (t >> 2)) * 8 + (t & 3); }

__host__ __device__ inline bool bits_ok(int b) { return b == 2 || b == 4 || b == 8; }

// Values of the codes of the paper's formats.  An IEEE-style format nests in a wider one: the magnitude bits of
// an E4M3 or E2M1 code, placed under the exponent of a binary16 number, are that number up to a power of two
// (subnormals included).
__device__ inline float e4m3_value(uint32_t b) {
  const uint16_t h = (uint16_t)(((b & 0x80u) << 8) | ((b & 0x7Fu) << 7));
  return (float)__builtin_bit_cast(_Float16, h) * 256.0f;
}
__device__ inline float e2m1_value(uint32_t n) {
  const uint16_t h = (uint16_t)(((n & 8u) << 12) | ((n & 7u) << 9));
  return (float)__builtin_bit_cast(_Float16, h) * 16384.0f;
}
__device__ inline float ternary_value(uint32_t c) { return (c & 1u) ? ((c & 2u) ? -1.0f : 1.0f) : 0.0f; }
// value of a code of the b-bit type of THINKV_FMT_FP, before its scale
__device__ inline float fp_code_value(uint32_t code, int bits) {
  return bits == 8 ? e4m3_value(code) : (bits == 4 ? e2m1_value(code) : ternary_value(code));
}

// index helpers for the per-(sequence, layer[, type]) tables
__device__ inline int64_t table_base(const thinkv_config& c, int seq, int layer, int cls) {
  return (((int64_t)seq * c.n_layers + layer) * 3 + cls) * (int64_t)c.max_pages;
}
__device__ inline int npages_index(const thinkv_config& c, int seq, int layer, int cls) {
  return (seq * c.n_layers + layer) * 3 + cls;
}
__device__ inline int sl_index(const thinkv_config& c, int seq, int layer) { return seq * c.n_layers + layer; }

// Soft eviction of one handle of sequence s (a valid sequence id).  The live bit is cleared with
// one atomic; only the thread that saw it set goes on to mark the slot reclaimable, so duplicates
// and dead slots count once.
__device__ inline void evict_one(const thinkv_view& v, int layer, int s, int32_t h) {
  const thinkv_config& c = v.cfg;
  if (h == -1) return;   // placeholder: no token
  const uint32_t uh = (uint32_t)h;
  const int cls = uh >> 28, pi = (uh >> 4) & 0xFFFFFF, slot = uh & 15;
  uint32_t* status = &v.dev_status[sl_index(c, s, layer)];
  if (h < 0 || cls > 2 || pi >= v.n_pages[npages_index(c, s, layer, cls)]) {
    atomicOr(status, THINKV_ST_BAD_SLOT);
    return;
  }
  uint32_t* mask = &v.slot_mask[table_base(c, s, layer, cls) + pi];
  const uint32_t bit = 1u << slot;
  const uint32_t old = atomicAnd(mask, ~bit);
  if (old & bit) {
    atomicOr(mask, bit << 16);
    atomicSub(&v.n_live[sl_index(c, s, layer)], 1);
  } else {
    atomicOr(status, THINKV_ST_EVICT_DEAD);
  }
}

// widen one element of a 16/32-bit float array exactly to binary32
__device__ inline float load_as_f32(const void* p, int64_t i, int dtype) {
  if (dtype == THINKV_F16) {
    return (float)(((const _Float16*)p)[i]);
  } else if (dtype == THINKV_BF16) {
    uint32_t u = ((uint32_t)((const uint16_t*)p)[i]) << 16;
    return __builtin_bit_cast(float, u);
  }
  return ((const float*)p)[i];
}

__device__ inline uint16_t f32_to_bf16_rne(float f) {
  uint32_t u = __builtin_bit_cast(uint32_t, f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40);  // NaN stays NaN
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

__device__ inline void store_from_f32(void* p, int64_t i, int dtype, float v) {
  if (dtype == THINKV_F16) {
    ((_Float16*)p)[i] = (_Float16)v;
  } else if (dtype == THINKV_BF16) {
    ((uint16_t*)p)[i] = f32_to_bf16_rne(v);
  } else {
    ((float*)p)[i] = v;
  }
}

}  // namespace thinkv
