// Pieces shared by the top-p kernels (register-resident per-head path and
// the multi-workgroup path for long candidate rows).
#pragma once
#include "tw_common.h"

constexpr uint32_t kKeyNegInf = 0x007FFFFFu;   // tw_float_key(-inf)

constexpr int HP_NB = 512;                     // histogram buckets per pass
constexpr uint32_t HP_FINE_END = 1u << 25;     // ranks below this (8 logits under the max) get the fine first pass
constexpr uint32_t HP_NONE = 0xFFFFFFFFu;      // rank of a score that takes no part (invalid slot or zero mass)
// Words that many workgroups update with atomics (head maxima, counters) sit 128 bytes apart:
// atomics to one cache line are served one after the other, whatever word they address.
constexpr int TW_CTR = 32;                     // stride in 32-bit words
// The long-row path's per-head maximum is folded by every scoring workgroup: spread over this
// many words per head (workgroup x folds into word x % HM_SLOTS); readers take the max of them.
constexpr int HM_SLOTS = 32;

// Workspace of twilight_topp_prune (byte offsets).  Both paths use scores,
// headmax, bitmaps, arrive; the rest belongs to the long-row path.
struct PruneWs {
  size_t scores, headmax, bitmaps, arrive, state, ghistM, ghistC, ulist, ucount, kdef, segcnt, total;
  int words_stride;       // bitmap words per head
};
PruneWs tw_prune_layout(const TwDims& d, int bound_pages, bool full);
PruneWs tw_prune_layout_tokens(const TwDims& d, int max_cand);   // token-list candidates (register-resident path only)

int tw_score_all_tokens_masked(const twilight_kv_t* kv, const TwDims& d, const void* q, const uint32_t* chmask, float* scores,
                               hipStream_t s);

// The pruner with the scoring - and, with `bounds`, the page selection - inside the per-head top-p kernel (per-head
// page lists, 4-bit codes, rows short enough for registers: tw_prune_fused_ok).  ws = a TW_WS_PRUNE workspace for
// this max_sel whose arrival counters (tw_prune_layout(d, max_sel, false).arrive, batch * Hkv * TW_CTR words) a
// kernel earlier on the stream has cleared.
bool tw_prune_fused_ok(const TwDims& d, int max_sel, bool with_select);
int tw_prune_fused(const twilight_kv_t* kv, const TwDims& d, const void* q, const float* bounds, const int32_t* budget,
                   int32_t* sel_pages, int32_t* sel_count, int32_t max_sel, float p, int32_t* kept_count, int32_t* kept_idx,
                   int32_t kept_stride, int32_t* union_count, int32_t* union_idx, int32_t union_stride,
                   uint32_t* status, void* ws, hipStream_t s);

#ifdef __HIPCC__
// softmax numerator e in [0, 1] -> floor(e * 2^40), exactly: the top 8 bits and the remaining 32
// bits are taken by two float -> integer truncations (every step below is exact in fp32: scaling by
// a power of two, the integer part of a value below 2^9, and the difference of the two)
__device__ __forceinline__ unsigned long long hp_fix(float e) {
  const float t = e * 256.0f;
  const uint32_t hi = (uint32_t)t;
  const float rem = t - (float)hi;
  const uint32_t lo = (uint32_t)(rem * 4294967296.0f);
  return ((unsigned long long)hi << 32) | lo;
}
// rank of a score: distance to the max logit in 2^-22 units; HP_NONE when the score is
// invalid or more than 27.5 logits below the max (its 2^-40 fixed-point mass is at most one unit there)
__device__ __forceinline__ uint32_t hp_rank_only(float m, float s) {
  const float d = __fsub_rn(m, s);
  return d < 27.5f ? (uint32_t)(d * 4194304.f) : HP_NONE;
}
__device__ __forceinline__ float hp_numer(float m, float s) { return __expf(-__fsub_rn(m, s)); }
__device__ __forceinline__ uint32_t hp_rank(float m, float s, float* e_out) {
  *e_out = hp_numer(m, s);
  return hp_rank_only(m, s);
}
#endif
