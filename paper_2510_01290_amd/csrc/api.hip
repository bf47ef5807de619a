// C ABI entry points: argument checks and kernel dispatch.  No allocation, no synchronisation; the
// only state is what never changes (the device's compute-unit count, the address of the
// library's own scratch array on each device).
#include <cstdlib>
#include "decode_common.h"

namespace thinkv {
size_t append_ws_bytes(const thinkv_config& c, int n_tok);
int launch_append(const thinkv_view& v, int layer, const void* k_new, const void* v_new, const int32_t* tok_seq,
                  const int32_t* tok_pos, const uint8_t* tok_class, int32_t* tok_handle, int n_tok, int in_dtype,
                  void* workspace, hipStream_t st, const int32_t* ev_seq, const int32_t* ev_handle, int n_ev);
int launch_evict(const thinkv_view& v, int layer, const int32_t* ev_seq, const int32_t* ev_handle, int n_ev, hipStream_t st);
int launch_init(const thinkv_view& v, hipStream_t st);
int launch_decode_simple(const thinkv_view& v, const DecodeArgs& a, hipStream_t st);
int launch_decode_mfma(const thinkv_view& v, const DecodeArgs& a, hipStream_t st);
size_t tbe_ws_bytes(const thinkv_config& c, int n_tok, int n_seg);
size_t tbe_plan_ws_bytes(int B, int max_cuts);
int launch_tbe_plan(const thinkv_view& v, int layer, const int32_t* seq_ids, const int32_t* seg_start, const uint8_t* seg_type,
                    const int32_t* n_segs, const uint8_t* transition_ended, int32_t* seg_count, int rule, int B, int max_segs, int budget, int max_cuts,
                    int cap_seg, int cap_tok, int32_t* tok_seq, int32_t* tok_handle, int32_t* seg_offset, int32_t* seg_keep,
                    int32_t* counts, void* workspace, hipStream_t st);
int launch_tbe_select(const thinkv_view& v, int layer, const int32_t* tok_seq, const int32_t* tok_handle, const int32_t* seg_offset,
                      const int32_t* seg_keep, int n_seg, int n_tok, int max_iters, int32_t* ev_handle, void* workspace,
                      hipStream_t st);
int launch_decode_mfma_stat(const thinkv_view& v, const DecodeArgs& a, hipStream_t st);
int launch_stat_fill(const thinkv_view& v, const DecodeArgs& a, hipStream_t st);
int launch_stat_count(const thinkv_view& v, const DecodeArgs& a, hipStream_t st);
int launch_decode_merge(const thinkv_view& v, const DecodeArgs& a, hipStream_t st);
int decode_mfma_supported(const thinkv_config& c);
int launch_gather_rows(const void* src, void* dst, const int32_t* rows, int64_t n_rows, int row_bytes, int n_wg, hipStream_t st);
int launch_probe_stream(const thinkv_view& v, int layer, const int32_t* seq_ids, int B, int per_head, uint32_t* checksum, hipStream_t st);


static int check_config(const thinkv_config* c) {
  if (!c) return THINKV_E_INVALID_ARG;
  if (c->page_size != kPage || c->group_size != kGroup) return THINKV_E_SHAPE;
  if (c->head_dim != 64 && c->head_dim != 128) return THINKV_E_SHAPE;
  if (c->n_layers < 1 || c->n_kv_heads < 1 || c->n_q_heads < 1 || c->max_seqs < 1 || c->max_pages < 1) return THINKV_E_SHAPE;
  if (c->n_q_heads % c->n_kv_heads) return THINKV_E_SHAPE;
  if (c->n_q_heads / c->n_kv_heads > 8) return THINKV_E_SHAPE;
  if (c->max_pages >= (1 << 24)) return THINKV_E_SHAPE;
  for (int k = 0; k < 3; ++k)
    if (!bits_ok(c->bits_of_class[k])) return THINKV_E_SHAPE;
  if (c->format != THINKV_FMT_INT && c->format != THINKV_FMT_FP) return THINKV_E_UNSUPPORTED;
  if (c->format == THINKV_FMT_FP)
    for (int k = 0; k < 2; ++k)
      if (!(c->fp8_scale[k] > 0.0f) || !(c->fp8_scale[k] < 3.0e38f)) return THINKV_E_INVALID_ARG;
  return THINKV_OK;
}

static int check_view(const thinkv_view* v) {
  if (!v) return THINKV_E_INVALID_ARG;
  int rc = check_config(&v->cfg);
  if (rc) return rc;
  for (int k = 0; k < 3; ++k) {
    if (v->arena_pages[k] < 0 || v->arena_pages[k] > 0x7fffffff) return THINKV_E_INVALID_ARG;
    if (v->arena_pages[k] > 0 && (!v->arena[k] || !v->free_stack[k] || !v->page_filled[k] || !v->slot_pos[k] || !v->page_pos_max[k]))
      return THINKV_E_INVALID_ARG;
  }
  if (!v->free_top || !v->block_table || !v->slot_mask || !v->n_pages || !v->n_live || !v->work_counters || !v->append_counters || !v->dev_status) return THINKV_E_INVALID_ARG;
  return THINKV_OK;
}

// Work-item sizes.  The fast kernel's items are single waves; the
// plain kernel's are workgroups of four waves, three to a compute unit (the fast kernel: two or three waves a SIMD, by head_dim).  An item pays a fixed
// price (query set-up, three type switches, its partial row), so it is given at least a few page
// pairs.  Where the launch has few (query, kv-head) pairs, the items of the longest sequence fill
// the machine exactly once; where it has many, an item per so many pages, about sixteen rounds of
// them if every sequence were as long as the host's bound: on full-attention layers the items of
// a head share its queues, so late items simply find less to do.
// A sliding-window layer is another matter: only the pages that hold one of the last W positions
// are worked on, the rest of the page list is merely scanned (a few bytes a page), so the fixed
// price of an item dominates: an item scans at least 64 pages per wave.
static int compute_units() {
  static int cached[64];
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) dev = 0;
  if (cached[dev] == 0) {
    int cus = 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0) cus = 256;
    cached[dev] = cus;
  }
  return cached[dev];
}

struct ItemSizing {
  int n_rows, per_head, ppi;
};

static ItemSizing size_items(const thinkv_config& c, int B, int max_ctx_pages, int window, bool fast) {
  const int64_t heads = (int64_t)B * c.n_kv_heads;
  const int64_t resident = fast ? (int64_t)compute_units() * 4 * decode_waves_per_simd(c.head_dim) : (int64_t)compute_units() * 3;
  const int least = window > 0 ? (fast ? 64 : 256) : (fast ? 16 : 32);   // fewest pages worth an item
  int64_t cap = ((int64_t)max_ctx_pages + least - 1) / least;
  if (cap < 1) cap = 1;
  if (cap > kMaxRowsPerHead) cap = kMaxRowsPerHead;
  int64_t per_head;
  if (window > 0)
    per_head = resident / heads;
  else if (heads * 2 <= resident)
    // all items resident at once; twice as many for larger batches, which are rarely of one length: an item per so many
    // pages then gives the longer contexts more workers than the shorter ones, and late items find what is left
    per_head = (B > 32 ? 2 : 1) * resident / heads;
  else
    per_head = ((fast ? 16 : 4) * resident + heads - 1) / heads;
  if (per_head > cap) per_head = cap;
  if (per_head < 1) per_head = 1;
  ItemSizing z;
  z.per_head = (int)per_head;
  z.n_rows = (int)(per_head * heads);
  z.ppi = (int)(((int64_t)max_ctx_pages + per_head - 1) / per_head);
  if (z.ppi < 1) z.ppi = 1;
  return z;
}

// partial rows any decode call with these bounds can need
static int64_t rows_bound(const thinkv_config& c, int B, int max_ctx_pages) {
  int64_t most = 1;
  for (int fast = 0; fast < 2; ++fast)
    for (int window = 0; window < 2; ++window) {
      const ItemSizing z = size_items(c, B, max_ctx_pages, window, fast != 0);
      if (z.n_rows > most) most = z.n_rows;
    }
  return most;
}

static size_t partial_bytes_of(const thinkv_config& c, int64_t rows) {
  const int G = c.n_q_heads / c.n_kv_heads;
  return (size_t)rows * G * (c.head_dim + kRowPad) * sizeof(float);
}

static int decode_common(const thinkv_view* view, int32_t layer, const void* q, void* out, float* lse,
                         const int32_t* seq_ids, const int32_t* q_pos, int32_t B, int32_t window, float softmax_scale,
                         int q_dtype, int out_dtype, int32_t max_ctx_pages, void* workspace, size_t workspace_bytes,
                         void* stream, bool fast, float* sparsity = nullptr) {
  int rc = check_view(view);
  if (rc) return rc;
  if (B < 0 || layer < 0 || layer >= view->cfg.n_layers || window < 0 || max_ctx_pages < 0) return THINKV_E_INVALID_ARG;
  if (B > view->cfg.max_seqs) return THINKV_E_INVALID_ARG;   // one row of work counters per query
  if (!(softmax_scale > 0.0f) || !(softmax_scale < 3.0e38f)) return THINKV_E_INVALID_ARG;   // also rejects NaN
  if (B == 0) return THINKV_OK;
  if (!q || !out || !seq_ids || !workspace || (window > 0 && !q_pos)) return THINKV_E_INVALID_ARG;
  if (q_dtype != THINKV_F16 && q_dtype != THINKV_BF16) return THINKV_E_UNSUPPORTED;
  if (out_dtype != THINKV_F16 && out_dtype != THINKV_BF16 && out_dtype != THINKV_F32) return THINKV_E_UNSUPPORTED;
  fast = fast && decode_mfma_supported(view->cfg);
  if (sparsity && !fast) return THINKV_E_UNSUPPORTED;
  const size_t partial_bytes = thinkv_decode_workspace_bytes(&view->cfg, B, max_ctx_pages);
  if (workspace_bytes < (sparsity ? thinkv_decode_sparsity_workspace_bytes(&view->cfg, B, max_ctx_pages) : partial_bytes)) return THINKV_E_WORKSPACE;
  DecodeArgs a;
  a.q = q;
  a.out = out;
  a.lse = lse;
  a.seq_ids = seq_ids;
  a.q_pos = q_pos;
  a.partial = (float*)workspace;
  a.layer = layer;
  a.B = B;
  a.window = window;
  a.q_dtype = q_dtype;
  a.out_dtype = out_dtype;
  const ItemSizing z = size_items(view->cfg, B, max_ctx_pages, window, fast);
  a.n_rows = z.n_rows;
  a.per_head = z.per_head;
  a.ppi = z.ppi;
  // the heads' first rows and row counts behind the partial rows
  a.alloc = (int32_t*)((char*)workspace + ((partial_bytes_of(view->cfg, rows_bound(view->cfg, B, max_ctx_pages)) + 255) & ~(size_t)255));
  a.scale_log2e = softmax_scale * 1.4426950408889634f;
  a.stat = nullptr;
  a.stat_stride = 0;
  a.sparsity = sparsity;
  a.direct = fast && !sparsity && a.per_head == 1;   // short contexts or huge batches: one item per head, no merge launch
  hipStream_t st = (hipStream_t)stream;
  if (sparsity) {
    // pooled scores behind the partials (whose size is a multiple of 16 bytes)
    a.stat = (float*)((char*)workspace + ((partial_bytes + 255) & ~(size_t)255));
    a.stat_stride = (int64_t)kPage * (max_ctx_pages > 0 ? max_ctx_pages : 1);
    rc = launch_stat_fill(*view, a, st);
    if (rc) return rc;
    rc = launch_decode_mfma_stat(*view, a, st);
    if (rc) return rc;
    rc = launch_decode_merge(*view, a, st);
    if (rc) return rc;
    return launch_stat_count(*view, a, st);
  }
  rc = fast ? launch_decode_mfma(*view, a, st) : launch_decode_simple(*view, a, st);
  if (rc || a.direct) return rc;
  return launch_decode_merge(*view, a, st);
}

}  // namespace thinkv

using namespace thinkv;

extern "C" {

size_t thinkv_block_bytes(const thinkv_config* cfg, int bits) {
  if (check_config(cfg) || !bits_ok(bits)) return 0;
  return (size_t)block_geom(bits, cfg->head_dim, cfg->format).block_bytes;
}

size_t thinkv_page_bytes(const thinkv_config* cfg, int bits) {
  return thinkv_block_bytes(cfg, bits) * (cfg ? (size_t)cfg->n_kv_heads : 0);
}

size_t thinkv_append_workspace_bytes(const thinkv_config* cfg, int32_t n_tok) {
  if (check_config(cfg) || n_tok < 0) return 0;
  return append_ws_bytes(*cfg, n_tok);
}

size_t thinkv_decode_workspace_bytes(const thinkv_config* cfg, int32_t B, int32_t max_ctx_pages) {
  if (check_config(cfg) || B < 0 || max_ctx_pages < 0) return 0;
  // partial rows, then two words per (query, kv-head)
  const int b1 = B > 0 ? B : 1;
  return ((partial_bytes_of(*cfg, rows_bound(*cfg, b1, max_ctx_pages)) + 255) & ~(size_t)255) + (size_t)b1 * cfg->n_kv_heads * 2 * sizeof(int32_t) + 256;
}

size_t thinkv_decode_sparsity_workspace_bytes(const thinkv_config* cfg, int32_t B, int32_t max_ctx_pages) {
  const size_t partial = thinkv_decode_workspace_bytes(cfg, B, max_ctx_pages);
  if (partial == 0) return 0;
  return ((partial + 255) & ~(size_t)255) +
         (size_t)(B > 0 ? B : 1) * cfg->n_kv_heads * (kPage * (size_t)(max_ctx_pages > 0 ? max_ctx_pages : 1) + 1) * sizeof(float);
}

int thinkv_init_view(const thinkv_view* view, void* stream) {
  int rc = check_view(view);
  if (rc) return rc;
  return launch_init(*view, (hipStream_t)stream);
}

int thinkv_append_quantized(const thinkv_view* view, int32_t layer, const void* k_new, const void* v_new,
                            const int32_t* tok_seq, const int32_t* tok_pos, const uint8_t* tok_class,
                            int32_t* tok_handle, int32_t n_tok, thinkv_dtype in_dtype, void* workspace,
                            size_t workspace_bytes, void* stream) {
  int rc = check_view(view);
  if (rc) return rc;
  if (n_tok < 0 || layer < 0 || layer >= view->cfg.n_layers) return THINKV_E_INVALID_ARG;
  if (n_tok == 0) return THINKV_OK;
  if (!k_new || !v_new || !tok_seq || !tok_pos || !tok_class || !workspace) return THINKV_E_INVALID_ARG;
  if (in_dtype != THINKV_F16 && in_dtype != THINKV_BF16 && in_dtype != THINKV_F32) return THINKV_E_UNSUPPORTED;
  if (workspace_bytes < append_ws_bytes(view->cfg, n_tok)) return THINKV_E_WORKSPACE;
  return launch_append(*view, layer, k_new, v_new, tok_seq, tok_pos, tok_class, tok_handle, n_tok, (int)in_dtype,
                       workspace, (hipStream_t)stream, nullptr, nullptr, 0);
}

int thinkv_evict_append(const thinkv_view* view, int32_t layer, const int32_t* ev_seq, const int32_t* ev_handle, int32_t n_ev,
                        const void* k_new, const void* v_new, const int32_t* tok_seq, const int32_t* tok_pos,
                        const uint8_t* tok_class, int32_t* tok_handle, int32_t n_tok, thinkv_dtype in_dtype, void* workspace,
                        size_t workspace_bytes, void* stream) {
  // a long eviction list (every plan workgroup reads all of it: one workgroup per sequence slot of the view), or no
  // tokens to append: the two calls one after the other
  if (n_tok <= 0 || n_ev <= 0 || n_ev > 4096 || (view && (int64_t)n_ev * view->cfg.max_seqs > (1 << 20))) {
    const int rc = thinkv_evict(view, layer, ev_seq, ev_handle, n_ev, stream);
    if (rc) return rc;
    return thinkv_append_quantized(view, layer, k_new, v_new, tok_seq, tok_pos, tok_class, tok_handle, n_tok, in_dtype, workspace,
                                   workspace_bytes, stream);
  }
  int rc = check_view(view);
  if (rc) return rc;
  if (layer < 0 || layer >= view->cfg.n_layers) return THINKV_E_INVALID_ARG;
  if (!ev_seq || !ev_handle || !k_new || !v_new || !tok_seq || !tok_pos || !tok_class || !workspace) return THINKV_E_INVALID_ARG;
  if (in_dtype != THINKV_F16 && in_dtype != THINKV_BF16 && in_dtype != THINKV_F32) return THINKV_E_UNSUPPORTED;
  if (workspace_bytes < append_ws_bytes(view->cfg, n_tok)) return THINKV_E_WORKSPACE;
  return launch_append(*view, layer, k_new, v_new, tok_seq, tok_pos, tok_class, tok_handle, n_tok, (int)in_dtype, workspace,
                       (hipStream_t)stream, ev_seq, ev_handle, n_ev);
}

int thinkv_evict(const thinkv_view* view, int32_t layer, const int32_t* ev_seq, const int32_t* ev_handle, int32_t n_ev,
                 void* stream) {
  int rc = check_view(view);
  if (rc) return rc;
  if (n_ev < 0 || layer < 0 || layer >= view->cfg.n_layers) return THINKV_E_INVALID_ARG;
  if (n_ev == 0) return THINKV_OK;
  if (!ev_seq || !ev_handle) return THINKV_E_INVALID_ARG;
  return launch_evict(*view, layer, ev_seq, ev_handle, n_ev, (hipStream_t)stream);
}

int thinkv_decode_attention(const thinkv_view* view, int32_t layer, const void* q, void* out, float* lse,
                            const int32_t* seq_ids, const int32_t* q_pos, int32_t B, int32_t window,
                            float softmax_scale, thinkv_dtype q_dtype, thinkv_dtype out_dtype, int32_t max_ctx_pages,
                            void* workspace, size_t workspace_bytes, void* stream) {
  return decode_common(view, layer, q, out, lse, seq_ids, q_pos, B, window, softmax_scale, (int)q_dtype, (int)out_dtype,
                       max_ctx_pages, workspace, workspace_bytes, stream, true);
}

// Partial rows of thinkv_decode_attention_noalloc.  In host code this name is only a stand-in for the
// symbol: the array's address on a device comes from hipGetSymbolAddress (once per device, below).
static __device__ __align__(256) unsigned char scratch[THINKV_NOALLOC_SCRATCH_BYTES];

int thinkv_decode_attention_noalloc(const thinkv_view* view, int32_t layer, const void* q, void* out, float* lse,
                                    const int32_t* seq_ids, const int32_t* q_pos, int32_t B, int32_t window,
                                    float softmax_scale, thinkv_dtype q_dtype, thinkv_dtype out_dtype,
                                    int32_t max_ctx_pages, void* stream) {
  static void* scratch_of_device[64];
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return THINKV_E_HIP;
  if (scratch_of_device[dev] == nullptr) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || p == nullptr) return THINKV_E_HIP;
    scratch_of_device[dev] = p;
  }
  if (view && B > 0 && max_ctx_pages >= 0 && check_config(&view->cfg) == THINKV_OK &&
      thinkv_decode_workspace_bytes(&view->cfg, B, max_ctx_pages) > (size_t)THINKV_NOALLOC_SCRATCH_BYTES)
    return THINKV_E_WORKSPACE;
  return decode_common(view, layer, q, out, lse, seq_ids, q_pos, B, window, softmax_scale, (int)q_dtype, (int)out_dtype,
                       max_ctx_pages, scratch_of_device[dev], (size_t)THINKV_NOALLOC_SCRATCH_BYTES, stream, true);
}

int thinkv_decode_attention_valu(const thinkv_view* view, int32_t layer, const void* q, void* out, float* lse,
                                 const int32_t* seq_ids, const int32_t* q_pos, int32_t B, int32_t window,
                                 float softmax_scale, thinkv_dtype q_dtype, thinkv_dtype out_dtype, int32_t max_ctx_pages,
                                 void* workspace, size_t workspace_bytes, void* stream) {
  return decode_common(view, layer, q, out, lse, seq_ids, q_pos, B, window, softmax_scale, (int)q_dtype, (int)out_dtype,
                       max_ctx_pages, workspace, workspace_bytes, stream, false);
}

int thinkv_decode_attention_sparsity(const thinkv_view* view, int32_t layer, const void* q, void* out, float* lse,
                                     float* sparsity, const int32_t* seq_ids, const int32_t* q_pos, int32_t B,
                                     int32_t window, float softmax_scale, thinkv_dtype q_dtype, thinkv_dtype out_dtype,
                                     int32_t max_ctx_pages, void* workspace, size_t workspace_bytes, void* stream) {
  if (!sparsity && B > 0) return THINKV_E_INVALID_ARG;
  return decode_common(view, layer, q, out, lse, seq_ids, q_pos, B, window, softmax_scale, (int)q_dtype, (int)out_dtype,
                       max_ctx_pages, workspace, workspace_bytes, stream, true, sparsity);
}

size_t thinkv_tbe_workspace_bytes(const thinkv_config* cfg, int32_t n_tok, int32_t n_seg) {
  if (check_config(cfg) || n_tok < 0 || n_seg < 0) return 0;
  return tbe_ws_bytes(*cfg, n_tok, n_seg);
}

int thinkv_tbe_select(const thinkv_view* view, int32_t layer, const int32_t* tok_seq, const int32_t* tok_handle,
                      const int32_t* seg_offset, const int32_t* seg_keep, int32_t n_seg, int32_t n_tok,
                      int32_t max_iters, int32_t* ev_handle, void* workspace, size_t workspace_bytes, void* stream) {
  int rc = check_view(view);
  if (rc) return rc;
  if (n_seg < 0 || n_tok < 0 || max_iters < 1 || layer < 0 || layer >= view->cfg.n_layers) return THINKV_E_INVALID_ARG;
  if (n_seg == 0 || n_tok == 0) return THINKV_OK;
  if (!tok_seq || !tok_handle || !seg_offset || !seg_keep || !ev_handle || !workspace) return THINKV_E_INVALID_ARG;
  if (workspace_bytes < tbe_ws_bytes(view->cfg, n_tok, n_seg)) return THINKV_E_WORKSPACE;
  return launch_tbe_select(*view, layer, tok_seq, tok_handle, seg_offset, seg_keep, n_seg, n_tok, max_iters, ev_handle,
                           workspace, (hipStream_t)stream);
}

size_t thinkv_tbe_plan_workspace_bytes(int32_t B, int32_t max_cuts) {
  if (B < 0 || max_cuts < 1) return 0;
  return tbe_plan_ws_bytes(B, max_cuts);
}

int thinkv_tbe_plan(const thinkv_view* view, int32_t layer, const int32_t* seq_ids, const int32_t* seg_start,
                    const uint8_t* seg_type, const int32_t* n_segs, const uint8_t* transition_ended, int32_t* seg_count, int32_t rule, int32_t B,
                    int32_t max_segs, int32_t budget, int32_t max_cuts, int32_t cap_seg, int32_t cap_tok,
                    int32_t* tok_seq, int32_t* tok_handle, int32_t* seg_offset, int32_t* seg_keep, int32_t* counts,
                    void* workspace, size_t workspace_bytes, void* stream) {
  int rc = check_view(view);
  if (rc) return rc;
  if (B < 0 || layer < 0 || layer >= view->cfg.n_layers || budget < 0 || cap_seg < 0 || cap_tok < 0) return THINKV_E_INVALID_ARG;
  if (max_segs < 1 || max_segs > THINKV_TBE_MAX_SEGS || max_cuts < 1 || max_cuts > THINKV_TBE_MAX_SEGMENT) return THINKV_E_INVALID_ARG;
  if (!seq_ids || !seg_start || !seg_type || !n_segs || !tok_seq || !tok_handle || !seg_offset || !seg_keep || !counts || !workspace)
    return THINKV_E_INVALID_ARG;
  if (rule != THINKV_TBE_BY_COUNT && rule != THINKV_TBE_BY_SIZE) return THINKV_E_INVALID_ARG;
  if (rule == THINKV_TBE_BY_COUNT && !seg_count) return THINKV_E_INVALID_ARG;
  if (workspace_bytes < tbe_plan_ws_bytes(B, max_cuts)) return THINKV_E_WORKSPACE;
  return launch_tbe_plan(*view, layer, seq_ids, seg_start, seg_type, n_segs, transition_ended, seg_count, rule, B, max_segs, budget, max_cuts,
                         cap_seg, cap_tok, tok_seq, tok_handle, seg_offset, seg_keep, counts, workspace, (hipStream_t)stream);
}

int thinkv_probe_stream_pages(const thinkv_view* view, int32_t layer, const int32_t* seq_ids, int32_t B, uint32_t* checksum, void* stream) {
  int rc = check_view(view);
  if (rc) return rc;
  if (B < 0 || layer < 0 || layer >= view->cfg.n_layers || B > view->cfg.max_seqs) return THINKV_E_INVALID_ARG;
  if (B == 0) return THINKV_OK;
  if (!seq_ids || !checksum) return THINKV_E_INVALID_ARG;
  // four waves to a workgroup, as many workgroups as fill the machine at the occupancy of the attention kernel
  int64_t per_head = (int64_t)compute_units() * decode_waves_per_simd(view->cfg.head_dim) / ((int64_t)B * view->cfg.n_kv_heads);
  if (per_head < 1) per_head = 1;
  return launch_probe_stream(*view, layer, seq_ids, B, (int)per_head, checksum, (hipStream_t)stream);
}

int thinkv_gather_rows(const void* src, void* dst, const int32_t* rows, int64_t n_rows, int32_t row_bytes, void* stream) {
  if (n_rows < 0 || row_bytes <= 0 || row_bytes % 16) return THINKV_E_INVALID_ARG;
  if (n_rows == 0) return THINKV_OK;
  if (!src || !dst || !rows) return THINKV_E_INVALID_ARG;
  if (((uintptr_t)src | (uintptr_t)dst) & 15) return THINKV_E_INVALID_ARG;
  const int64_t pieces = n_rows * (row_bytes / 16);
  int64_t n_wg = (pieces + 1023) / 1024;                      // four pieces a thread
  const int64_t most = (int64_t)compute_units() * 16;        // a few rounds of workgroups at most: the loop does the rest
  if (n_wg > most) n_wg = most;
  return launch_gather_rows(src, dst, rows, n_rows, row_bytes, (int)n_wg, (hipStream_t)stream);
}

const char* thinkv_status_string(int status) {
  switch (status) {
    case THINKV_OK: return "ok";
    case THINKV_E_INVALID_ARG: return "invalid argument";
    case THINKV_E_SHAPE: return "unsupported geometry";
    case THINKV_E_UNSUPPORTED: return "unsupported dtype or option";
    case THINKV_E_WORKSPACE: return "workspace too small";
    case THINKV_E_HIP: return "HIP call failed";
  }
  return "unknown status";
}

}  // extern "C"
