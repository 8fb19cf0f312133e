/*
 * twilight.h - C ABI of the MI355X (gfx950) Twilight decode hot path.
 *
 * One decode step of one attention layer (paper: Figure 5, Section 4.1):
 *
 *   twilight_kquant_append   new K/V rows -> paged bf16 pools, INT4 K copy
 *                            (Section 4.2; Appendix B.1), per-page key bounds
 *   twilight_select_pages    token selector: top pages by a per-page upper
 *                            bound of q.k (Section 4, challenge C1; Sec. 4.1)
 *   twilight_topp_prune      Twilight pruner: INT4 scores, softmax, top-p
 *                            threshold, per-group union (Sec. 4.2, Alg. 1,
 *                            Definition 3.3, Appendix B.2)
 *   twilight_sparse_decode   attention over the kept tokens (Definition 3.1,
 *                            Appendix B.2), split along the list with a
 *                            log-sum-exp combine
 *
 * Conventions
 *   - Every pointer is a DEVICE pointer unless its comment says "host".
 *     `stream` is a hipStream_t passed as void* (NULL = default stream).
 *   - The caller owns every buffer.  The library allocates nothing, frees
 *     nothing, copies nothing between host and device and never synchronises;
 *     all work is enqueued on `stream`.  It keeps no state between calls
 *     beyond cached device properties (compute-unit count, occupancy of its
 *     own kernels) and reads no environment variables; entry points may be
 *     called from several threads.  The one exception is the opt-in per-kernel
 *     timing of twilight_prof.h, which is process-global (off by default).
 *   - head_dim must be 128, page_size 16, quant_group 32, quant_bits 0/4, 2 or 8,
 *     num_q_heads / num_kv_heads one of 1, 2, 4, 8.
 *     (The kernels are compiled per group size: the heads of a group share
 *     every loaded bound, code page and K/V row in registers; at 16 heads per
 *     KV head the accumulators no longer fit a workgroup's registers, and a
 *     split into two passes of 8 would change the shape of the per-KV-head
 *     union lists.  Larger ratios are refused with TW_EINVAL.)
 *   - Query head h reads KV head h / (num_q_heads / num_kv_heads).
 *   - Size limits (TW_EINVAL beyond them): batch * num_q_heads <= 65535;
 *     num_pool_pages * num_kv_heads * 16 < 2^31; at most 2^22 candidate
 *     tokens per query head in twilight_topp_prune (max_sel * 16, or
 *     max_pages_per_seq * 16 with sel_pages == NULL), at most 8192 per row
 *     of a token list (the *_tokens entry points); batch * num_kv_heads
 *     (batch * num_q_heads for the per-head variant) <= 12000 in
 *     twilight_sparse_decode.
 *   - Token indices are logical positions in their sequence (0 .. len-1);
 *     page ids are logical page numbers (token / 16); both ascending in every
 *     list.  Pool addresses are resolved through page_table in the kernels.
 *     A page_table entry outside [0, num_pool_pages) is skipped (its tokens
 *     score -inf / are not written) - no out-of-bounds access is made.
 *   - Return value: TW_OK (0) or a negative TW_E* code for problems the host
 *     can see (NULL pointer, unsupported shape, workspace too small, launch
 *     failure).  Data-dependent conditions set bits in the device `status`
 *     word where an entry point has one.
 */
#ifndef TWILIGHT_H
#define TWILIGHT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define TW_ABI_VERSION 1

#define TW_OK 0
#define TW_EINVAL (-1)     /* NULL pointer, unsupported shape or parameter */
#define TW_EWORKSPACE (-2) /* workspace smaller than twilight_workspace_bytes */
#define TW_ELAUNCH (-3)    /* HIP reported an error (kernel launch, device or symbol query) */
#define TW_ELIMIT (-4)     /* problem larger than the fixed scratch of twilight_select_pages_static */

/* status bits (device word) */
#define TW_STATUS_UNION_TRUNCATED 1u /* a group's union exceeded union_stride */
#define TW_STATUS_KEPT_TRUNCATED 2u  /* a head's kept list exceeded kept_stride */

/*
 * Paged KV cache of one layer.  Layouts (all row-major, page = 16 tokens):
 *   k_pool, v_pool  bf16 [num_pool_pages][num_kv_heads][16][128]
 *   kq_pool         u8   [num_pool_pages][num_kv_heads][16][16 * quant_bits]
 *                   codes 0..2^quant_bits-1 of K (quant_bits = 4: the method's
 *                   INT4 copy, 64 bytes per token).  32-bit little-endian words:
 *                   4 bits: dims 8w..8w+7 form word w (w = 0..15); byte k
 *                           (k = 0..3) holds code[8w+k] in the low nibble and
 *                           code[8w+k+4] in the high nibble.
 *                   2 bits: dims 16w..16w+15 form word w (w = 0..7); byte i
 *                           holds code[16w+4k+i] at bits 2k..2k+1, k = 0..3.
 *                   8 bits: dims 4w..4w+3 form word w (w = 0..31), byte i =
 *                           code[4w+i].
 *                   The 2- and 8-bit copies are the other widths of the
 *                   paper's bit-width study of the estimator (Section 4.2).
 *   kq_meta         fp16 [num_pool_pages][num_kv_heads][16][4][2]
 *                   (scale, zero) of each group of 32 dims:
 *                   K ~ code * scale + zero           (Appendix B.1)
 *   page_minmax     bf16 [num_pool_pages][num_kv_heads][2][128]
 *                   element-wise (min, max) of K over the page's valid tokens
 *   page_table      i32  [batch][max_pages_per_seq]  logical page -> pool page
 *   seq_lens        i32  [batch]  tokens valid in the cache
 */
typedef struct twilight_kv {
  int32_t batch;
  int32_t num_q_heads;
  int32_t num_kv_heads;
  int32_t head_dim;          /* 128 */
  int32_t page_size;         /* 16  */
  int32_t quant_group;       /* 32  */
  int32_t max_pages_per_seq; /* row length of page_table */
  int32_t quant_bits;        /* width of the kq_pool codes: 4 (0 means 4), 2 or 8 */
  int64_t num_pool_pages;
  const int32_t* page_table;
  const int32_t* seq_lens;
  void* k_pool;
  void* v_pool;
  void* kq_pool;
  void* kq_meta;
  void* page_minmax;
} twilight_kv_t;

/*
 * Append new tokens (stage 4; Section 4.2: the additional asymmetric INT4
 * copy of K; Appendix B.1: quantised when written, fp16 scale and zero).
 * For sequence b the n_new[b] rows starting at row
 * new_offsets[b] of k_new / v_new become tokens start_pos[b] ..
 * start_pos[b]+n_new[b]-1.  Written: k_pool, v_pool (bf16 copies), kq_pool,
 * kq_meta, page_minmax of every page touched.  A page that already holds
 * tokens below start_pos[b] keeps their contribution to page_minmax (which
 * must be valid); otherwise its bounds are rebuilt from the new tokens.
 * seq_lens is NOT read or written (the caller advances it).
 *
 * Quantisation, per token, KV head and group of 32 dims, fp32 arithmetic,
 * every operation rounded on its own:
 *   scale = fp16((max - min) * (1/L)),  zero = fp16(min),  L = 2^quant_bits - 1 (15),
 *   code  = clamp(rint((x - zero) * (1 / scale)), 0, L)    (0 if scale == 0).
 * Inputs must be finite with |x| < 3e4 (fp16 range of scale and zero).
 *
 *   k_new, v_new   bf16 [total_new][num_kv_heads][128]; v_new may be NULL
 *                  (V pool untouched).  kv->k_pool may be NULL (no bf16 copy).
 *   start_pos, n_new, new_offsets   i32 [batch]
 *   max_new        host: upper bound of n_new[] (sizes the launch)
 */
int twilight_kquant_append(const twilight_kv_t* kv, const void* k_new, const void* v_new,
                           const int32_t* start_pos, const int32_t* n_new, const int32_t* new_offsets,
                           int32_t max_new, void* stream);

/*
 * Token selector (stage 1; Section 4.1: the base algorithm picks a generous
 * candidate set; Section 4, challenge C1: pooling per page of 16 tokens).  For every
 * (sequence, query head): U[P] = sum_d max(q_d*min[P,d], q_d*max[P,d]) in
 * fp32 - 16 partial sums of 8 consecutive dims each, left to right, then a
 * pairwise tree over the partials - and the Kp = min(ceil(budget/16), pages)
 * pages with the largest U are kept; equal U: lower page id first.
 *
 *   q              bf16 [batch][num_q_heads][128]
 *   budget_tokens  i32  [batch]
 *   sel_pages      i32  [batch][num_q_heads][max_sel]  out, ascending ids
 *   sel_count      i32  [batch][num_q_heads]           out, min(Kp, max_sel)
 *   ws             >= twilight_workspace_bytes(TW_WS_SELECT, ...)
 */
int twilight_select_pages(const twilight_kv_t* kv, const void* q, const int32_t* budget_tokens,
                          int32_t* sel_pages, int32_t* sel_count, int32_t max_sel,
                          void* ws, size_t ws_bytes, void* stream);

/*
 * twilight_select_pages for callers that cannot allocate device memory or hand
 * over a workspace: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same kernels, same results bit for bit;
 * the fp32 bound scores (batch * num_q_heads * max_pages_per_seq * 4 bytes) go
 * to a fixed array of TW_STATIC_SELECT_WS_BYTES of device memory that is part
 * of the library's code object (each GPU the library runs on holds its copy
 * until the process ends).  The call allocates and frees nothing (no hipMalloc /
 * hipFree, no allocating library routine; per-kernel timing must be off).
 * TW_ELIMIT when the scores do not fit; TW_ELAUNCH when the array's device
 * address cannot be obtained.  All calls on one GPU share the array, which
 * keeps the previous call's contents (every score that is read is written
 * first, so nothing needs clearing): calls that overlap on one GPU - on
 * different streams or from different threads - race and must be serialised
 * by the caller.
 */
#define TW_STATIC_SELECT_WS_BYTES (8u << 20)
int twilight_select_pages_static(const twilight_kv_t* kv, const void* q, const int32_t* budget_tokens,
                                 int32_t* sel_pages, int32_t* sel_count, int32_t max_sel, void* stream);

/*
 * The decode step's form of stages 4 + 1 in one launch: append ONE new token
 * per sequence (as twilight_kquant_append with n_new = 1 would: bf16 K/V rows,
 * INT4 codes, scale/zero, page bounds - bit for bit the same), then select
 * pages as twilight_select_pages does, the new token's page included.  Saves
 * the separate append launch of a decode step (any quant_bits).
 *   k_new, v_new   bf16 [batch][num_kv_heads][128] (v_new may be NULL; kv->k_pool
 *                  may be NULL as in twilight_kquant_append)
 *   new_pos        i32 [batch] position of the new token, < seq_lens[b]
 *                  (seq_lens already counts it); negative: nothing appended
 *                  for that sequence
 *   the rest       as twilight_select_pages
 */
int twilight_append_select(const twilight_kv_t* kv, const void* k_new, const void* v_new, const int32_t* new_pos,
                           const void* q, const int32_t* budget_tokens,
                           int32_t* sel_pages, int32_t* sel_count, int32_t max_sel,
                           void* ws, size_t ws_bytes, void* stream);

/*
 * Selector and pruner of a decode step in one call (Section 4.1: the token
 * selector's subset handed straight to the pruner; Section 4.2, Algorithm 1):
 * what twilight_append_select (k_new given) or twilight_select_pages (k_new,
 * v_new, new_pos all NULL) followed by twilight_topp_prune over the selected
 * pages computes - the same cache update, page lists, kept sets and unions,
 * bit for bit.  Where a head's list is short enough for one workgroup
 * (quant_bits = 4, max_sel <= 512 pages, sequences of at most 196608 tokens,
 * and not just a few heads with more than 4096 candidates each) the call is
 * two launches instead of four: the bounds of all pages, then one workgroup
 * per query head that picks the head's pages (sequences of at most 4096 pages;
 * longer ones keep the selection launch), scores their tokens from the
 * quantised K copy, runs top-p and, as the last head of its group, lists the
 * union.  Otherwise it runs the launches of the separate calls.  The
 * workspace needs no initialising.
 *   sel_pages, sel_count   out, as twilight_select_pages
 *   kept_count ... status  out, as twilight_topp_prune
 *   ws             >= twilight_workspace_bytes(TW_WS_SELECT_PRUNE, kv, max_sel, 0)
 *                  (the sizes of TW_WS_SELECT and TW_WS_PRUNE added)
 */
int twilight_select_prune(const twilight_kv_t* kv, const void* k_new, const void* v_new, const int32_t* new_pos,
                          const void* q, const int32_t* budget_tokens, float p,
                          int32_t* sel_pages, int32_t* sel_count, int32_t max_sel,
                          int32_t* kept_count, int32_t* kept_idx, int32_t kept_stride,
                          int32_t* union_count, int32_t* union_idx, int32_t union_stride,
                          uint32_t* status, void* ws, size_t ws_bytes, void* stream);

/*
 * Estimated scores alone (first half of stage 2; Section 4.2: the sparse
 * matrix-vector product over the quantised K copy; Appendix B.1).  q is quantised per head to int8 (sq = max|q| * (1/127),
 * qi = clamp(rint(q / sq), -127, 127)); per token and group j of 32 dims
 * I_j = sum qi_d * code_d (int32), Qs_j = sum qi_d;
 *   s_hat = ((T0 + T1) + (T2 + T3)) * (sq * (1/sqrt(128))),
 *   T_j   = fl(scale_j * float(I_j)) + fl(zero_j * float(Qs_j))   (fp32).
 * Candidate slot c of head (b, h) is token sel_pages[b][h][c / 16] * 16 +
 * c % 16; slots at or beyond seq_lens[b] score -inf.
 *
 *   sel_pages      NULL = every page of the sequence (then max_sel is
 *                  ignored and the row length is max_pages_per_seq * 16)
 *   scores         fp32 [batch][num_q_heads][max_sel * 16]            out
 *   dots           i32  [batch][num_q_heads][max_sel * 16][4] or NULL out
 */
int twilight_int4_score(const twilight_kv_t* kv, const void* q, const int32_t* sel_pages,
                        const int32_t* sel_count, int32_t max_sel, float* scores, int32_t* dots,
                        void* stream);

/*
 * Twilight pruner (stage 2; Section 4.2, Algorithm 1, Definition 3.3,
 * Appendix B.2).  Per (sequence, query head): s_hat as above over the
 * candidates, W = softmax(s_hat) over the candidates, tau* = the largest
 * weight value whose upper set {W >= tau*} has mass >= p, kept = that upper
 * set (all ties at the cut).  The threshold is found with histograms of the
 * softmax mass over the distance to the largest score (masses in 64-bit fixed
 * point, so the result does not depend on the order of accumulation) and an
 * exact comparison of the last few candidates on the bits of s_hat.
 * p >= 1 keeps every candidate.  Per (sequence, KV head): union = sorted
 * unique union of the kept sets of its query heads.
 *
 *   sel_pages/sel_count/max_sel   as in twilight_int4_score (NULL = all)
 *   p              host, in (0, 1]
 *   kept_count     i32 [batch][num_q_heads]               out
 *   kept_idx       i32 [batch][num_q_heads][kept_stride]  out or NULL
 *   union_count    i32 [batch * num_kv_heads]             out
 *   union_idx      i32 [batch * num_kv_heads][union_stride] out, ascending
 *   status         u32 device word, OR-ed with TW_STATUS_* bits; lists are
 *                  then cut after their first stride entries (counts too)
 *   ws             >= twilight_workspace_bytes(TW_WS_PRUNE, ...)
 */
int twilight_topp_prune(const twilight_kv_t* kv, const void* q, const int32_t* sel_pages,
                        const int32_t* sel_count, int32_t max_sel, float p,
                        int32_t* kept_count, int32_t* kept_idx, int32_t kept_stride,
                        int32_t* union_count, int32_t* union_idx, int32_t union_stride,
                        uint32_t* status, void* ws, size_t ws_bytes, void* stream);

/*
 * The pruner behind ANY token-level selector (Section 4.1: the base algorithm
 * is a black box that hands over a token subset I_0; Section 4.2 then prunes
 * it).  Same arithmetic and the same outputs as twilight_int4_score /
 * twilight_topp_prune, but the candidates of a query head are a list of token
 * positions instead of a list of pages: candidate slot c of head (b, h) is
 * token cand_tokens[b][h][c].
 *
 *   cand_tokens    i32 [batch][num_q_heads][max_cand], ascending, distinct.
 *                  Entries outside [0, seq_lens[b]) or on unmapped pages score
 *                  -inf and are never kept.
 *   cand_count     i32 [batch][num_q_heads], clamped to [0, max_cand]
 *   max_cand       host: a multiple of 16, at most 8192; the sequences must
 *                  not exceed 196608 tokens (max_pages_per_seq * 16)
 *   scores         fp32 [batch][num_q_heads][max_cand]           out
 *   dots           i32  [batch][num_q_heads][max_cand][4] or NULL out
 *   ws             >= twilight_workspace_bytes(TW_WS_PRUNE_TOKENS, kv, max_cand, 0)
 *   the rest       as twilight_topp_prune
 */
int twilight_int4_score_tokens(const twilight_kv_t* kv, const void* q, const int32_t* cand_tokens,
                               const int32_t* cand_count, int32_t max_cand, float* scores, int32_t* dots,
                               void* stream);
int twilight_topp_prune_tokens(const twilight_kv_t* kv, const void* q, const int32_t* cand_tokens,
                               const int32_t* cand_count, int32_t max_cand, float p,
                               int32_t* kept_count, int32_t* kept_idx, int32_t kept_stride,
                               int32_t* union_count, int32_t* union_idx, int32_t union_stride,
                               uint32_t* status, void* ws, size_t ws_bytes, void* stream);

/*
 * A second token selector for the front of the pruner, of the channel-sparse
 * kind (Section 4.1: the base algorithm is a black box; Sections 4.3 and 5
 * name a Double-Sparsity-style selector, which ranks tokens by an estimate
 * taken from a few channels of a 4-bit copy of K - the copy this cache
 * already holds).  The paper does not define that selector; the form built
 * here: per KV head a fixed set of channels (found offline by the caller),
 * per (sequence, query head) the estimate of EVERY token of the sequence,
 *   s_ds = the s_hat of twilight_int4_score with the int8 query set to 0
 *          outside the channel set (sq stays that of the whole query),
 * and the min(budget, length, max_cand) tokens with the largest estimate are
 * handed over; equal estimates: lower position first.  The lists feed
 * twilight_topp_prune_tokens (max_cand <= 8192 there).
 *
 *   channel_mask   u32 [num_kv_heads][4]: bit (d % 32) of word d / 32 set =
 *                  channel d of that KV head takes part
 *   budget_tokens  i32 [batch]
 *   cand_tokens    i32 [batch][num_q_heads][max_cand]  out, ascending positions
 *   cand_count     i32 [batch][num_q_heads]            out
 *   ws             >= twilight_workspace_bytes(TW_WS_DS_SELECT, kv, max_cand, 0)
 *                  (one fp32 estimate per token and query head)
 */
int twilight_ds_select_tokens(const twilight_kv_t* kv, const void* q, const uint32_t* channel_mask,
                              const int32_t* budget_tokens, int32_t* cand_tokens, int32_t* cand_count,
                              int32_t max_cand, void* ws, size_t ws_bytes, void* stream);

/*
 * Sparse decode attention (stage 3; Definition 3.1 with the weights
 * renormalised over the attended set, Appendix B.2 group-wise varlen).
 * Every query head of KV head g attends over union_idx[b*Hkv+g][0..count):
 *   out = sum_t softmax_t(q.K_t / sqrt(128)) V_t      bf16 in, fp32 math.
 * The list is split into chunks handled by different workgroups; partial
 * (max, sum, accumulator) triples are merged by log-sum-exp.
 *
 *   union_idx      NULL = dense attention over all seq_lens[b] tokens
 *                  (union_count and union_stride are then ignored).  Entries
 *                  outside [0, seq_lens[b]) and entries on unmapped pages are
 *                  skipped; an entry listed twice counts twice.
 *   out            bf16 [batch][num_q_heads][128]
 *   lse            fp32 [batch][num_q_heads] or NULL: natural-log
 *                  log-sum-exp of the scaled logits (-inf for an empty set,
 *                  whose output row is 0)
 *   ws             >= twilight_workspace_bytes(TW_WS_DECODE, ...)
 */
int twilight_sparse_decode(const twilight_kv_t* kv, const void* q, const int32_t* union_count,
                           const int32_t* union_idx, int32_t union_stride, void* out, float* lse,
                           void* ws, size_t ws_bytes, void* stream);

/*
 * The head-wise variable-length alternative of Appendix B.2: every query head
 * attends over its OWN kept set instead of its group's union (same
 * arithmetic, one list per query head; the K/V rows of a KV head are then
 * loaded once per query head that kept them instead of once per group).
 *   kept_count     i32 [batch][num_q_heads]
 *   kept_idx       i32 [batch][num_q_heads][kept_stride], ascending token
 *                  positions, as written by twilight_topp_prune
 *   ws             >= twilight_workspace_bytes(TW_WS_DECODE_PER_HEAD, kv, 0, kept_stride)
 */
int twilight_sparse_decode_per_head(const twilight_kv_t* kv, const void* q, const int32_t* kept_count,
                                    const int32_t* kept_idx, int32_t kept_stride, void* out, float* lse,
                                    void* ws, size_t ws_bytes, void* stream);

/* Workspace sizes (host-only query; no GPU needed). */
#define TW_WS_SELECT 0
#define TW_WS_PRUNE 1
#define TW_WS_DECODE 2
#define TW_WS_DECODE_PER_HEAD 3
#define TW_WS_PRUNE_TOKENS 4
#define TW_WS_DS_SELECT 5
#define TW_WS_SELECT_PRUNE 6
/*  max_sel: as passed to the call (0 with sel_pages == NULL; max_cand for
 *  TW_WS_PRUNE_TOKENS);
 *  union_stride: as passed to sparse_decode (0 for dense), kept_stride for
 *  TW_WS_DECODE_PER_HEAD. */
size_t twilight_workspace_bytes(int which, const twilight_kv_t* kv, int32_t max_sel, int32_t union_stride);

/*
 * Offloaded KV cache (the paper's offloading scenario, its appendix on
 * efficiency with the KV cache in CPU memory): k_pool / v_pool may live in
 * PINNED HOST memory (hipHostMalloc); the kernels then fetch only the rows of
 * the kept tokens over the host link, while the quantised K copy, its
 * scale/zero and the page bounds stay in device memory.  This call returns
 * the device-side address of such an allocation (hipHostGetDevicePointer) for
 * use in twilight_kv_t; TW_EINVAL if host_ptr (host) is not mapped pinned memory.
 */
int twilight_pinned_device_pointer(void* host_ptr, void** device_ptr /* host, out */);

const char* twilight_strerror(int code);
int twilight_abi_version(void);

#ifdef __cplusplus
}
#endif
#endif /* TWILIGHT_H */
