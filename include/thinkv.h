/*
 * thinkv.h -- C ABI of the ThinKV decode hot path for AMD MI355X (gfx950).
 *
 * A paged KV cache whose tokens are group-quantised at a precision chosen by their thought
 * type, whose evicted tokens are only marked in a mask, and whose freed slots are reused in
 * place by newly appended tokens of the same type (the paper's "Continuous Thinking" memory
 * manager, Sec. 5.2, with thought-adaptive quantisation, Sec. 4.2), plus decode-step grouped-
 * query attention computed directly over the packed pages (appendix "Decode", "Grouped-Query
 * Attention"; physical slot order is irrelevant by the theorem "KV Permutation Invariance of
 * Attention").
 *
 * Conventions
 *   - Every pointer inside thinkv_view and every array argument marked DEVICE is device
 *     memory owned by the caller; the library allocates nothing and keeps no global state.
 *   - Every call enqueues work on the caller's HIP stream and returns without synchronising.
 *     Calls on one view must be ordered by the stream(s) the caller uses.
 *   - Return value: a thinkv_status for problems the host can see (null pointers, bad
 *     geometry, workspace too small, launch failure).  Problems only the device can see set
 *     bit flags in view->dev_status and skip the offending token / slot; nothing aborts.
 *   - Thought types are numbered as in the paper's pseudocode: 0 = transition (T),
 *     1 = execution (E), 2 = reasoning (R).  bits_of_class maps a type to 2, 4 or 8 bits.
 */
#ifndef THINKV_H
#define THINKV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { THINKV_F16 = 0, THINKV_BF16 = 1, THINKV_F32 = 2 } thinkv_dtype;

typedef enum {
  THINKV_OK = 0,
  THINKV_E_INVALID_ARG = 1, /* null pointer, negative count, bad enum                      */
  THINKV_E_SHAPE = 2,       /* geometry the kernels do not cover                            */
  THINKV_E_UNSUPPORTED = 3, /* dtype / option combination not implemented                   */
  THINKV_E_WORKSPACE = 4,   /* workspace_bytes smaller than thinkv_*_workspace_bytes()      */
  THINKV_E_HIP = 5          /* a HIP call or kernel launch failed                           */
} thinkv_status;

/* bit flags in dev_status[seq * n_layers + layer]; the last word of dev_status
 * (index max_seqs * n_layers) collects conditions that belong to no valid sequence. */
#define THINKV_ST_NOPAGES 1u    /* page pool of the class empty, or the page list full       */
#define THINKV_ST_BAD_CLASS 2u  /* tok_class > 2                                             */
#define THINKV_ST_BAD_SLOT 4u   /* evict handle names no page of that sequence               */
#define THINKV_ST_EVICT_DEAD 8u /* evict of a slot that holds no live token (ignored)        */
#define THINKV_ST_BAD_SEQ 16u   /* sequence id outside [0, max_seqs)                         */
#define THINKV_ST_BAD_SEGMENT 32u /* thinkv_tbe_select: segment larger than THINKV_TBE_MAX_SEGMENT or
                                    keep outside 1..THINKV_TBE_MAX_KEEP; nothing of it is evicted */

#define THINKV_PAGE_SIZE 16
#define THINKV_TBE_MAX_SEGMENT 256 /* live tokens of one segment handed to thinkv_tbe_select */
#define THINKV_TBE_MAX_KEEP 64     /* largest retention level (the paper's schedule starts at 64) */
#define THINKV_TBE_MAX_SEGS 2048   /* segments of one sequence thinkv_tbe_plan looks at          */
#define THINKV_TBE_BY_COUNT 0      /* thinkv_tbe_plan: retention level from the segment's selection count */
#define THINKV_TBE_BY_SIZE 1       /* thinkv_tbe_plan: retention level from the segment's live size       */
#define THINKV_GROUP_SIZE 32

/* Static geometry; host memory, passed by value inside thinkv_view. */
typedef struct {
  int32_t n_layers, n_q_heads, n_kv_heads;
  int32_t head_dim;         /* 64 or 128                                                     */
  int32_t page_size;        /* 16 slots per page                                             */
  int32_t group_size;       /* 32 consecutive channels share a scale and zero-point          */
  int32_t bits_of_class[3]; /* each 2, 4 or 8; index = thought type                          */
  int32_t max_seqs;
  int32_t max_pages;        /* capacity of each (sequence, layer, type) page list            */
  int32_t format;           /* THINKV_FMT_INT (0) or THINKV_FMT_FP                           */
  float fp8_scale[2];       /* THINKV_FMT_FP: the per-tensor scales of keys and of values of
                               the 8-bit (E4M3) type, positive, from calibration             */
} thinkv_config;

/*
 * Number formats of the cache.
 *   THINKV_FMT_INT  asymmetric integer codes (appendix "Group Quantization"): groups of 32 channels of a
 *                   token share a binary16 scale and zero-point; x^ = zp + code * scale.  The bench format.
 *   THINKV_FMT_FP   the paper's own formats (Sec. 4.2, appendix "Quantization Data Formats"), chosen by the
 *                   type's bit width: 8 = FP8 E4M3 (finite-only, bias 7) with the per-tensor scale above;
 *                   4 = NVFP4: E2M1 codes (bias 1; sign in bit 3) with one E4M3 scale per 16 channels of
 *                   the token; 2 = ternary (bit 1 sign, bit 0 magnitude; -0 never written) with one E4M3
 *                   scale per 16 channels.  x^ = value(code) * scale; no zero-points.  Codes round to
 *                   nearest, ties to the even code, and saturate; a group's scale is amax / qmax
 *                   (qmax 6 / 1) rounded up to the next E4M3 value.  Code regions of a block are laid out
 *                   as for THINKV_FMT_INT; a meta region is head_dim/16 * 16 scale bytes, byte
 *                   group16 * 16 + slot (none for the 8-bit type).  Every call works in either format.
 */
#define THINKV_FMT_INT 0
#define THINKV_FMT_FP 1

/*
 * The cache.  The paper's block table (physical block #, # filled, thought type, eviction
 * mask; Sec. 5.2 "Block Table") is kept as one page list per (sequence, layer, thought type)
 * -- the table sorted by its thought-type column -- plus per-physical-page state:
 *
 *   arena[c]        packed pages of type c, page stride thinkv_page_bytes(cfg, bits_of_class[c])
 *   free_stack[c]   [arena_pages[c]] LIFO pool; free_top[c] = number of free pages
 *   block_table     [max_seqs][n_layers][3][max_pages] physical page numbers, -1 = unused
 *   n_pages         [max_seqs][n_layers][3]
 *   page_filled[c]  [arena_pages[c]] slots ever written, 0..16 (the paper's "# Filled")
 *   slot_mask       [max_seqs][n_layers][3][max_pages], parallel to block_table (the table's
 *                   "eviction mask" column): bits 0..15: slot holds a live token; bits 16..31:
 *                   slot soft-evicted and reclaimable.  Kept in list order so that attention and
 *                   append read the masks of a page list as one contiguous run.
 *   slot_pos[c]     [arena_pages[c]][16] logical position of the token in the slot, -1 = none
 *   page_pos_max[c] [arena_pages[c]] an upper bound of the page's slot_pos entries: the largest
 *                   position ever written into the page (-1 = none).  Sliding-window attention
 *                   skips pages whose bound lies before the window without reading slot_pos.
 *   n_live          [max_seqs][n_layers] live tokens
 *   work_counters   [n_layers][max_seqs][n_kv_heads][4] scratch of thinkv_decode_attention: per
 *                   (layer, query index, kv-head) the heads of three work queues (one per type)
 *                   and a spare word; zero between calls (init zeroes them, every call leaves
 *                   them zero), so two decode calls on one (view, layer) must not overlap
 *   append_counters [max_seqs] scratch of thinkv_append_quantized (arrival counts of the
 *                   workgroups of a sequence); zero between calls
 *   dev_status      [max_seqs * n_layers + 1] THINKV_ST_* flags
 *
 * Byte layout of one page: n_kv_heads blocks of thinkv_block_bytes(); a block is
 * [K codes: 64 chunks of CB = (head_dim/32)*b bytes][K meta][V codes: 64 chunks][V meta];
 * a meta region is NG*4 units (NG = head_dim/32) of eight binary16: unit group*4 + slot/4 holds
 * the scales of its four slots (slot%4 = 0..3), then their four zero-points.
 * Inside a chunk a b-bit code sits at
 * bit 32*(f / FPH) + 16*h + b*(f % FPH), FPH = 16/b, with
 *   K, slot t, channel c: chunk 16*((c%32)/8) + t, f = 4*(c/32) + (c%8)/2, h = c%2
 *   V, slot t, channel c: chunk 16*(t/4) + c%16,   f = ((t%4)/2)*(head_dim/16) + c/16, h = t%2
 */
typedef struct {
  thinkv_config cfg;
  uint8_t* arena[3];        /* DEVICE */
  int64_t arena_pages[3];
  int32_t* free_stack[3];   /* DEVICE */
  int32_t* free_top;        /* DEVICE [3] */
  int32_t* block_table;     /* DEVICE */
  int32_t* n_pages;         /* DEVICE */
  uint8_t* page_filled[3];  /* DEVICE */
  uint32_t* slot_mask;      /* DEVICE */
  int32_t* slot_pos[3];     /* DEVICE */
  int32_t* page_pos_max[3]; /* DEVICE */
  int32_t* n_live;          /* DEVICE */
  uint32_t* work_counters;  /* DEVICE */
  uint32_t* append_counters;/* DEVICE */
  uint32_t* dev_status;     /* DEVICE */
} thinkv_view;

/* A slot handle names a slot of one sequence and layer: (type << 28) | (index in that type's
 * page list << 4) | slot.  thinkv_append_quantized reports the handle each token received. */
#define THINKV_HANDLE(type, page_idx, slot) (((int32_t)(type) << 28) | ((int32_t)(page_idx) << 4) | (int32_t)(slot))

/* Layout queries (host, pure).  Return 0 for unsupported geometry. */
size_t thinkv_block_bytes(const thinkv_config* cfg, int bits); /* one (page, kv-head)        */
size_t thinkv_page_bytes(const thinkv_config* cfg, int bits);  /* n_kv_heads blocks          */

/* Bytes of scratch thinkv_append_quantized needs for a call with n_tok tokens. */
size_t thinkv_append_workspace_bytes(const thinkv_config* cfg, int32_t n_tok);
/* Bytes of scratch thinkv_decode_attention needs for B queries when no sequence holds more
 * than max_ctx_pages pages (summed over the three types) in the layer attended.  The launch is
 * sized for the machine, so the answer depends on the compute-unit count of the CURRENT device
 * (256 is assumed where there is none): ask with the device current on which the call will run. */
size_t thinkv_decode_workspace_bytes(const thinkv_config* cfg, int32_t B, int32_t max_ctx_pages);

/* Puts a view into the empty state: free stacks filled so that pages come out 0,1,2,...,
 * tables -1, counters and flags 0, slot_pos and page_pos_max -1, arenas zero-filled (attention reads the
 * never-written slots of a partly filled page and discards them by their live bit, so their
 * scales and zero-points have to be finite numbers).  arena[c] must be 16-byte aligned. */
int thinkv_init_view(const thinkv_view* view, void* stream /* hipStream_t */);

/*
 * Quantise-and-append (paper Sec. 4.2 Problem "Thought-Adaptive Quantization": each new KV
 * entry is quantised at the precision of its thought type; Sec. 5.2 "Efficient Memory
 * Management" and the appendix walkthrough, step d: the token goes to a reclaimable slot of an
 * existing block of its type, else to the next unused slot of the last block of that type,
 * else to a newly allocated block; never into a block of another type).
 *
 *   k_new, v_new  DEVICE [n_tok][n_kv_heads][head_dim] of in_dtype (post-RoPE keys)
 *   tok_seq       DEVICE [n_tok] sequence ids, non-decreasing
 *   tok_pos       DEVICE [n_tok] logical positions
 *   tok_class     DEVICE [n_tok] thought types
 *   tok_handle    DEVICE [n_tok] out, may be NULL: handle of each token, -1 if it was skipped
 *
 * Tokens of one sequence are applied in array order; among reclaimable slots the first page
 * in list order and its lowest slot go first; new pages are popped in token order, so the
 * result equals a one-token-at-a-time loop.  Quantiser: per group of 32 channels, zero-point =
 * binary16(min), scale = smallest binary16 >= (max-min)/(2^b-1), code = clamp(rint((x-zp)/
 * scale), 0, 2^b-1) in binary32 with IEEE division and round-half-even.
 * Skipped tokens: invalid sequence or type, or no page available (flags in dev_status).
 * No alignment is required of k_new and v_new; calls of more than 64 tokens are faster when both
 * are 16-byte aligned.
 */
int thinkv_append_quantized(const thinkv_view* view, int32_t layer, const void* k_new, const void* v_new,
                            const int32_t* tok_seq, const int32_t* tok_pos, const uint8_t* tok_class,
                            int32_t* tok_handle, int32_t n_tok, thinkv_dtype in_dtype, void* workspace,
                            size_t workspace_bytes, void* stream);

/*
 * Soft eviction (paper Sec. 5.2 "TBE with CT": evicted tokens are only marked in the
 * eviction mask; removal is deferred until a new token overwrites the slot).
 *   ev_seq, ev_handle  DEVICE [n_ev]
 * Sets the slot's reclaimable bit, clears its live bit, decrements n_live.  A handle whose slot
 * holds no live token is ignored (THINKV_ST_EVICT_DEAD); duplicates in one call count once.
 * A handle of -1 (what append reports for a token it could not place, and what
 * thinkv_tbe_select writes for a survivor) is skipped without a flag.
 */
int thinkv_evict(const thinkv_view* view, int32_t layer, const int32_t* ev_seq, const int32_t* ev_handle,
                 int32_t n_ev, void* stream);

/*
 * The two calls of a decode step in one (Sec. 5.2: a step marks the tokens its eviction policy
 * chose and the newly generated token takes a freed slot): the same result, tables, bytes and
 * flags as thinkv_evict(ev_seq, ev_handle, n_ev) followed by thinkv_append_quantized(...) with
 * the same arguments, with one kernel launch less (the evictions of a sequence are applied by
 * the workgroup that plans the sequence's appends).
 */
int thinkv_evict_append(const thinkv_view* view, int32_t layer, const int32_t* ev_seq, const int32_t* ev_handle, int32_t n_ev,
                        const void* k_new, const void* v_new, const int32_t* tok_seq, const int32_t* tok_pos,
                        const uint8_t* tok_class, int32_t* tok_handle, int32_t n_tok, thinkv_dtype in_dtype, void* workspace,
                        size_t workspace_bytes, void* stream);

/*
 * Decode attention (appendix "Decode": O = softmax(q K^T / sqrt(d)) V over every cached
 * token; "Grouped-Query Attention": the n_q_heads / n_kv_heads query heads of a group share
 * one K/V head, each with its own softmax).  K^ and V^ are zp + code * scale from the stored
 * binary16 scale and zero-point; slots whose live bit is clear are not attended; with window
 * W > 0 only slots with 0 <= q_pos - slot_pos < W are.
 *
 *   q        DEVICE [B][n_q_heads][head_dim] of q_dtype (F16 or BF16)
 *   out      DEVICE [B][n_q_heads][head_dim] of out_dtype
 *   lse      DEVICE [B][n_q_heads] float, may be NULL: log-sum-exp of the scaled scores
 *   seq_ids  DEVICE [B] which sequence each query belongs to; B <= max_seqs
 *   q_pos    DEVICE [B] logical position of the query (used only when window > 0)
 *   max_ctx_pages  host upper bound on pages (all types) any attended sequence holds; it sizes the launch and the
 *                  workspace.  A sequence that holds more is still attended in full, by fewer workers than it would get.
 *
 * A query with no visible token gets out = 0 and lse = -inf.  Accumulation is binary32.
 */
int thinkv_decode_attention(const thinkv_view* view, int32_t layer, const void* q, void* out, float* lse,
                            const int32_t* seq_ids, const int32_t* q_pos, int32_t B, int32_t window,
                            float softmax_scale, thinkv_dtype q_dtype, thinkv_dtype out_dtype,
                            int32_t max_ctx_pages, void* workspace, size_t workspace_bytes, void* stream);

/*
 * thinkv_decode_attention for callers that cannot allocate device memory or hand over a
 * workspace: code running under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same contract, arguments and kernels as thinkv_decode_attention, minus the
 * workspace: the partial rows live in an array of THINKV_NOALLOC_SCRATCH_BYTES that is part of the
 * library's device image (every GPU the library runs on holds its own copy until the process ends).
 * The call allocates and frees nothing.  Launches whose partial rows do not fit (ask
 * thinkv_decode_workspace_bytes with the same B and max_ctx_pages) return THINKV_E_WORKSPACE.
 * All calls of a process on one GPU share that GPU's array: two calls that overlap in time on one
 * GPU (different streams) race; calls on one stream are ordered and safe.  Nothing in the array
 * needs clearing between calls (every word read was written by the same call).
 */
#define THINKV_NOALLOC_SCRATCH_BYTES (32u << 20)
int thinkv_decode_attention_noalloc(const thinkv_view* view, int32_t layer, const void* q, void* out, float* lse,
                                    const int32_t* seq_ids, const int32_t* q_pos, int32_t B, int32_t window,
                                    float softmax_scale, thinkv_dtype q_dtype, thinkv_dtype out_dtype,
                                    int32_t max_ctx_pages, void* stream);

/* Same contract and arguments as thinkv_decode_attention, computed by the plain vector-ALU
 * kernel (binary32 dequantisation, no matrix cores).  Kept as a slow cross-check. */
int thinkv_decode_attention_valu(const thinkv_view* view, int32_t layer, const void* q, void* out, float* lse,
                                 const int32_t* seq_ids, const int32_t* q_pos, int32_t B, int32_t window,
                                 float softmax_scale, thinkv_dtype q_dtype, thinkv_dtype out_dtype,
                                 int32_t max_ctx_pages, void* workspace, size_t workspace_bytes, void* stream);

/*
 * Thought-adaptive eviction, the choice of survivors (Sec. 4.3 "Think Before you Evict" and
 * appendix "TBE Eviction Policy"): a thought segment picked for eviction is cut down to
 * K = min(|segment|, keep) tokens by K-means over its keys; of every cluster the member nearest
 * the centroid survives, with its value.  The paper fixes no K-means variant; this one is
 * Lloyd's algorithm on the stored keys, dequantised, all kv-heads of a token concatenated, tokens
 * in the order listed: initial centroid j = point floor(j*N/K); assign to the nearest centroid
 * (squared distance, ties to the lowest cluster); stop when no assignment changed or after
 * max_iters assignments, else move the centroids to the means of their points (an emptied
 * cluster keeps its centroid); survivors = per non-empty cluster the nearest member (ties to the
 * lowest index; of two members the earlier one).  At most K tokens of a segment survive.
 * Which segments are cut, and to what size (the paper's Case 1 / Case 2 and retention schedule
 * {64,32,16,8,4}), is the caller's decision and arrives as seg_keep.
 *
 *   tok_seq, tok_handle  DEVICE [n_tok] the live tokens of the segments, segment after segment,
 *                        inside a segment in ascending position; all tokens of a segment belong
 *                        to one sequence
 *   seg_offset           DEVICE [n_seg + 1] segment s owns tokens [seg_offset[s], seg_offset[s+1]),
 *                        at most THINKV_TBE_MAX_SEGMENT of them
 *   seg_keep             DEVICE [n_seg] tokens to retain, 1..THINKV_TBE_MAX_KEEP
 *   ev_handle            DEVICE [n_tok] out: the token's handle if it is to be evicted, -1 if it
 *                        survives -- ready for thinkv_evict(view, layer, tok_seq, ev_handle, n_tok),
 *                        which skips entries of -1
 *   workspace            at least thinkv_tbe_workspace_bytes(cfg, n_tok, n_seg).  On return it holds, from its first
 *                        256-byte boundary on: float x[n_tok][n_kv_heads * head_dim], the dequantised keys;
 *                        float cent[n_seg][THINKV_TBE_MAX_KEEP][n_kv_heads * head_dim], the centroids after the last
 *                        update; int32 assign[n_tok], every token's cluster at the last assignment (-1 where the
 *                        segment was not clustered) -- for callers that want to inspect the clustering
 * Arithmetic is binary32 (products of 22-bit operands), squared distances taken as |x|^2 - 2 x.c + |c|^2; a decision between
 * two candidates whose distances differ by less than about 1e-5 of the points' mean squared norm
 * may differ from a binary64 evaluation.  Device-side errors: THINKV_ST_BAD_SLOT / BAD_SEQ for a token that
 * does not exist (it clusters as the origin and is never evicted), THINKV_ST_BAD_SEGMENT (in the
 * last word of dev_status) for a segment outside the limits (nothing of it is evicted).
 */
size_t thinkv_tbe_workspace_bytes(const thinkv_config* cfg, int32_t n_tok, int32_t n_seg);

/*
 * Thought-adaptive eviction, the plan (Sec. 4.3): which segments of the examined sequences are
 * cut now, and to how many tokens; the output is the input of thinkv_tbe_select.
 * Case 1: where transition_ended[b] is set (a transition segment of the sequence has just
 * ended), every preceding segment is selected.  Case 2: while the sequence holds more than
 * `budget` live tokens, the oldest segment of the least important type (0 = transition, then
 * 1 = execution, then 2 = reasoning) that can still be selected is.
 * What a selection does (problem statement "Thought-Adaptive Eviction" of Sec. 4.3, retention
 * schedule R = {64,32,16,8,4}):
 *   THINKV_TBE_BY_COUNT  the paper's rule.  seg_count[seq][segment] = n, how often the segment has been
 *                        selected so far; the selection keeps min(live tokens, R_n) and makes the count n + 1;
 *                        a segment can be selected while n < 5.  A selection that removes nothing is not listed
 *                        as a cut, it only advances the count.  The caller keeps the table (zero for a new segment).
 *   THINKV_TBE_BY_SIZE   for callers that keep no counts: the level follows from the segment's live
 *                        size, which is cut to the largest schedule value below it; seg_count is not used.
 * A segment is cut at most once per call; the last (open) segment is never touched; a segment
 * with more than THINKV_TBE_MAX_SEGMENT live tokens is left alone and reported
 * (THINKV_ST_BAD_SEGMENT in the last word of dev_status).  A cut that does not fit the output
 * lists is not made: its segment's count stays.
 * A live token belongs to the segment whose start is the largest one not above its position
 * (the block table's start-index column, Sec. 5.2 "Block Table").
 *
 *   seq_ids           DEVICE [B] sequences to examine (each at most once)
 *   seg_start         DEVICE [max_seqs][max_segs] first position of every segment of a sequence,
 *                     ascending; row = sequence id.  max_segs <= THINKV_TBE_MAX_SEGS
 *   seg_type          DEVICE [max_seqs][max_segs] thought type of the segment
 *   n_segs            DEVICE [max_seqs] segments the sequence has so far
 *   transition_ended  DEVICE [B], may be NULL (no Case 1 anywhere)
 *   seg_count         DEVICE [max_seqs][max_segs] in/out (THINKV_TBE_BY_COUNT; may be NULL under BY_SIZE)
 *   rule              THINKV_TBE_BY_COUNT or THINKV_TBE_BY_SIZE
 *   max_cuts          cuts per sequence and call at most (1..256); what is left waits for the next call
 *   cap_seg, cap_tok  capacity of the output lists; cuts that no longer fit are left for the next call
 *   tok_seq, tok_handle  DEVICE [cap_tok] out: the live tokens of the cut segments, segment after
 *                     segment, ascending position inside a segment
 *   seg_offset        DEVICE [cap_seg + 1] out; seg_keep DEVICE [cap_seg] out
 *   counts            DEVICE [2] out: number of cuts, number of listed tokens (the n_seg and n_tok
 *                     of the thinkv_tbe_select call that follows)
 *   workspace         at least thinkv_tbe_plan_workspace_bytes(B, max_cuts)
 */
size_t thinkv_tbe_plan_workspace_bytes(int32_t B, int32_t max_cuts);
int thinkv_tbe_plan(const thinkv_view* view, int32_t layer, const int32_t* seq_ids, const int32_t* seg_start,
                    const uint8_t* seg_type, const int32_t* n_segs, const uint8_t* transition_ended, int32_t* seg_count, int32_t rule, int32_t B,
                    int32_t max_segs, int32_t budget, int32_t max_cuts, int32_t cap_seg, int32_t cap_tok,
                    int32_t* tok_seq, int32_t* tok_handle, int32_t* seg_offset, int32_t* seg_keep, int32_t* counts,
                    void* workspace, size_t workspace_bytes, void* stream);
int thinkv_tbe_select(const thinkv_view* view, int32_t layer, const int32_t* tok_seq, const int32_t* tok_handle,
                      const int32_t* seg_offset, const int32_t* seg_keep, int32_t n_seg, int32_t n_tok,
                      int32_t max_iters, int32_t* ev_handle, void* workspace, size_t workspace_bytes, void* stream);

/*
 * Decode attention plus the attention-sparsity statistic of the step, from which the paper reads
 * the thought type (Sec. 4.1: the normalised attention scores of a decode step, an entry being
 * negligible below 1 % of its row's maximum; appendix "Grouped-Query Attention": per group of
 * query heads the scaled scores q_{h,g} . k^_j * softmax_scale are max-pooled over the G heads,
 * the pooled row is renormalised by a softmax over the keys, and the fractions of negligible
 * entries are averaged over the groups).  The keys are the same visible live set as for the
 * attention output.
 *
 *   sparsity   DEVICE [B] float, not NULL: mean over kv-heads of
 *              #{ j : softmax(pooled)_j < 0.01 * max_j softmax(pooled)_j } / #visible tokens,
 *              0 where nothing is visible.  Scores are binary32; an entry within rounding of the
 *              boundary may fall on either side.
 *   workspace  at least thinkv_decode_sparsity_workspace_bytes(cfg, B, max_ctx_pages): the pooled
 *              score of every slot is kept between the kernels, 64 bytes per page and kv-head.
 *              Sequences longer than max_ctx_pages pages are counted over their first
 *              max_ctx_pages pages only.
 * Everything else as thinkv_decode_attention, which this call otherwise equals (same out, lse).
 * The thresholds that turn the statistic into a thought type come from calibration and stay
 * with the caller.  Needs head_dim 64 or 128 and at most 8 query heads per kv-head
 * (THINKV_E_UNSUPPORTED otherwise).
 */
size_t thinkv_decode_sparsity_workspace_bytes(const thinkv_config* cfg, int32_t B, int32_t max_ctx_pages);
int thinkv_decode_attention_sparsity(const thinkv_view* view, int32_t layer, const void* q, void* out, float* lse,
                                     float* sparsity, const int32_t* seq_ids, const int32_t* q_pos, int32_t B,
                                     int32_t window, float softmax_scale, thinkv_dtype q_dtype,
                                     thinkv_dtype out_dtype, int32_t max_ctx_pages, void* workspace,
                                     size_t workspace_bytes, void* stream);

/*
 * Measurement aid (no part of the method): reads every (page, kv-head) block of the listed
 * sequences' page lists of one layer -- exactly the cache bytes a full-attention
 * thinkv_decode_attention call over the same sequences reads -- with plain streaming loads and no
 * arithmetic, split over the machine the way the attention launch is.  Its duration is what the
 * memory system gives for this layout.  checksum: DEVICE one word (any value; only ever xor-ed).
 */
int thinkv_probe_stream_pages(const thinkv_view* view, int32_t layer, const int32_t* seq_ids, int32_t B, uint32_t* checksum,
                              void* stream);

/*
 * Contrast, not part of the method: the gather a CONTIGUOUS cache needs after every eviction (Sec. 5.1
 * "The Cost of Gather-Based Compaction", Observations 4a / 4b) -- the data movement that in-place slot
 * reuse does without.  dst[i] = src[rows[i]] for i < n_rows, rows of row_bytes bytes.
 *   src   DEVICE rows of row_bytes bytes (16-byte aligned; row_bytes a multiple of 16)
 *   dst   DEVICE n_rows rows, must not overlap src
 *   rows  DEVICE [n_rows] indices into src (for a compaction: the surviving rows, ascending)
 */
int thinkv_gather_rows(const void* src, void* dst, const int32_t* rows, int64_t n_rows, int32_t row_bytes, void* stream);

const char* thinkv_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* THINKV_H */
