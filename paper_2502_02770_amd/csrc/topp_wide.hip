// Stage 2b/c for long candidate rows (paper: Algorithm 1, Definition 3.3,
// Appendix B.2): the same threshold search as the register-resident kernel,
// spread over many workgroups per head.  Used when a head has more than 8192
// candidates (every token a candidate - no selector in front - or very large
// budgets) or the sequence is too long for the in-LDS bitmap.
//
//   wide_init     clears histograms / lists / bitmaps, resets per-head state
//   (int4_score   also folds the row maximum into headmax with atomicMax)
//   wide_hist     one pass over the scores: LDS histogram of the current rank
//                 interval per workgroup, flushed to the head's global one
//   wide_decide   one wave per head scans the 2048 buckets and narrows the
//                 interval (or finishes when <= 4096 scores are left in it,
//                 which one pass achieves on rows of a million smooth scores)
//   wide_emit     second pass: kept for sure -> bitmap, undecided -> a short
//                 per-head list
//   wide_resolve  finish on the undecided list inside one workgroup (narrowing
//                 in LDS, then exact on the scores' own bits), sets their bits
//   bitmap_list   bitmap(s) -> ascending index list (per-head kept list, and
//                 the union of a KV head's query heads)
// All sums are 64-bit fixed point and all atomics are integer adds / maxima,
// so results do not depend on scheduling.
#include <stdlib.h>
#include "topp_common.h"

namespace {

struct WideState {           // per head
  uint32_t rlo, shift, pop, flags, pass, mk;    // mk: key of the head's largest score (0 = none), set by the first decide
  unsigned long long A, target;
};
constexpr uint32_t WF_DONE = 1, WF_EMPTY = 4, WF_TIER_ALL = 8;
constexpr int W_SLOTS = 32;                    // candidate slots per thread
constexpr int W_CAP = 4096;                    // undecided scores that the resolve kernel takes
constexpr int W_NB = 2048;                     // buckets per pass: pass 0 covers every rank (32 logits at 1/64)
constexpr int W_BITS = 11;

struct WideArgs {
  const float* scores;
  const int32_t* sel_pages;   // or nullptr
  const int32_t* sel_count;
  const int32_t* seq_lens;
  const uint32_t* headmax;    // [bh][HM_SLOTS] (padded): max = key of the head's largest score, 0 = no valid score
  WideState* state;
  unsigned long long* ghistM;
  uint32_t* ghistC;
  uint2* ulist;               // [bh][W_CAP] {key, token}
  uint32_t* ucount;
  uint32_t* kdef;
  uint32_t* bitmaps;
  int32_t* kept_count;
  uint32_t* status;
  int Hq, max_pages, max_sel, cand_stride, words_stride;
  int keep_all;               // p >= 1
  float p;
};

__global__ __launch_bounds__(256) void wide_init_kernel(uint4* zero_base, size_t n16, WideState* st, int nbh) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n16) zero_base[i] = make_uint4(0, 0, 0, 0);
  if (i < (size_t)nbh) {
    WideState s;
    s.rlo = 0; s.shift = 16; s.pop = 0; s.flags = 0; s.pass = 0; s.mk = 0; s.A = 0; s.target = 0;
    st[i] = s;
  }
}

// the head's largest score: maximum over the words the scoring workgroups folded into
__device__ __forceinline__ uint32_t wide_headmax(const uint32_t* headmax, int bh, int lane) {
  const uint32_t v = lane < HM_SLOTS ? headmax[((long long)bh * HM_SLOTS + lane) * TW_CTR] : 0u;
  return tw_wave_max_u32(v);
}

__device__ __forceinline__ int wide_count(const WideArgs& a, int b, int bh) {
  const int n = a.seq_lens[b];
  int P = n > 0 ? (n + TW_PAGE - 1) / TW_PAGE : 0;
  if (P > a.max_pages) P = a.max_pages;
  int count = P;
  if (a.sel_pages) { count = a.sel_count[bh]; if (count > a.max_sel) count = a.max_sel; if (count < 0) count = 0; }
  return count;
}

// A workgroup of NT threads covers NT * W_SLOTS consecutive candidate slots; thread t owns 8 groups
// of 4 slots, group v at chunk + v * 4 * NT + 4t, so that every load instruction of a wave reads
// 1 KiB contiguous.  Loaded unconditionally (clamped) and masked to -inf at and beyond N.
template <int NT>
__device__ __forceinline__ int wide_slot(int chunk0, int v, int tid) { return chunk0 + v * 4 * NT + tid * 4; }
template <int NT>
__device__ __forceinline__ void wide_load(const float* row, int chunk0, int tid, int N, int cand_stride, float* s) {
#pragma unroll
  for (int v = 0; v < W_SLOTS / 4; ++v) {
    const int c = wide_slot<NT>(chunk0, v, tid);
    const float4 x = *(const float4*)(row + (c < cand_stride ? c : cand_stride - 4));
    s[4 * v] = c < N ? x.x : -__builtin_inff();     // N is a multiple of 16: a group is inside or outside
    s[4 * v + 1] = c < N ? x.y : -__builtin_inff();
    s[4 * v + 2] = c < N ? x.z : -__builtin_inff();
    s[4 * v + 3] = c < N ? x.w : -__builtin_inff();
  }
}

template <int NT>
__global__ __launch_bounds__(NT) void wide_hist_kernel(WideArgs a) {
  constexpr int W_CHUNK = NT * W_SLOTS;
  const int bh = blockIdx.y, b = bh / a.Hq, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const WideState st = a.state[bh];
  if (st.flags & WF_DONE) return;
  const int N = wide_count(a, b, bh) * TW_PAGE;
  if ((long long)blockIdx.x * W_CHUNK >= N) return;
  const uint32_t mk = wide_headmax(a.headmax, bh, lane);
  if (mk == 0) return;
  const float m = tw_key_to_float(mk);
  const int chunk0 = blockIdx.x * W_CHUNK;

  __shared__ unsigned long long histM[W_NB];
  __shared__ uint32_t histC[W_NB];
  for (int i = tid; i < W_NB; i += NT) { histM[i] = 0; histC[i] = 0; }
  float s[W_SLOTS];
  wide_load<NT>(a.scores + (long long)bh * a.cand_stride, chunk0, tid, N, a.cand_stride, s);
  __syncthreads();
#pragma unroll
  for (int e = 0; e < W_SLOTS; ++e) {
    const uint32_t r = hp_rank_only(m, s[e]);       // the exponential only for scores that take part
    if (r != HP_NONE && r >= st.rlo) {
      const uint32_t bk = (r - st.rlo) >> st.shift;
      if (bk < W_NB) {
        atomicAdd(&histM[bk], hp_fix(hp_numer(m, s[e])));
        atomicAdd(&histC[bk], 1u);
      }
    }
  }
  __syncthreads();
  for (int i = tid; i < W_NB; i += NT) {
    const uint32_t c = histC[i];
    if (c) { atomicAdd(&a.ghistM[(long long)bh * W_NB + i], histM[i]); atomicAdd(&a.ghistC[(long long)bh * W_NB + i], c); }
  }
}

// One wave per head: scan the 2048 buckets (lane l owns 32l .. 32l+31), find the one where the
// mass reaches the target, narrow the interval to it.
__global__ __launch_bounds__(64) void wide_decide_kernel(WideArgs a) {
  constexpr int BPL = W_NB / 64;
  const int bh = blockIdx.x, lane = threadIdx.x;
  WideState st = a.state[bh];
  if (st.flags & WF_DONE) return;
  st.mk = wide_headmax(a.headmax, bh, lane);
  if (st.mk == 0) { if (lane == 0) { st.flags = WF_DONE | WF_EMPTY; a.state[bh] = st; } return; }
  unsigned long long* gm = a.ghistM + (long long)bh * W_NB;
  uint32_t* gc = a.ghistC + (long long)bh * W_NB;
  unsigned long long mb[BPL], mine = 0;
#pragma unroll
  for (int k = 0; k < BPL; ++k) { mb[k] = gm[BPL * lane + k]; mine += mb[k]; }
  const unsigned long long incl = tw_wave_scan_u64(mine);
  const unsigned long long total = __shfl(incl, 63, 64);
  if (st.pass == 0) {                             // pass 0 sees every score that has mass: total = Z
    const double t = ceil((double)a.p * (double)total);
    st.target = t < 1.0 ? 1ull : (unsigned long long)t;
    if (st.target > total) st.target = total;
  }
  const unsigned long long before = st.A + incl - mine;
  const bool hit = before < st.target && before + mine >= st.target;
  const unsigned long long bal = __ballot(hit);
  bool again = false;
  if (bal == 0) {
    st.flags |= WF_DONE | WF_TIER_ALL;            // unreachable: the interval holds the crossing by construction
  } else {
    const int src = __ffsll((long long)bal) - 1;
    unsigned long long cum = before, asel = before;
    int bsel = 0;
#pragma unroll
    for (int k = 0; k < BPL; ++k) {
      if (cum < st.target && cum + mb[k] >= st.target) { bsel = k; asel = cum; }
      cum += mb[k];
    }
    const int bucket = BPL * src + __shfl(bsel, src, 64);
    st.A = __shfl(asel, src, 64);
    st.pop = gc[bucket];
    st.rlo += (uint32_t)bucket << st.shift;
    if (st.pop <= (uint32_t)W_CAP) st.flags |= WF_DONE;
    else if (st.shift == 0) st.flags |= WF_DONE | WF_TIER_ALL;   // > W_CAP scores of one rank: keep them all
    else { st.shift = st.shift >= W_BITS ? st.shift - W_BITS : 0; again = true; }
  }
  st.pass += 1;
  if (again) {
#pragma unroll
    for (int k = 0; k < BPL; ++k) { gm[BPL * lane + k] = 0; gc[BPL * lane + k] = 0; }
  }
  if (lane == 0) a.state[bh] = st;
}

template <int NT>
__global__ __launch_bounds__(NT) void wide_emit_kernel(WideArgs a) {
  constexpr int W_CHUNK = NT * W_SLOTS;
  const int bh = blockIdx.y, b = bh / a.Hq, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const WideState st = a.state[bh];
  if (!a.keep_all && st.mk == 0) return;          // no valid score: bitmap stays empty
  const int count = wide_count(a, b, bh);
  const int N = count * TW_PAGE;
  if ((long long)blockIdx.x * W_CHUNK >= N) return;
  const float m = tw_key_to_float(st.mk);
  const int chunk0 = blockIdx.x * W_CHUNK;
  // a search that did not finish in the passes given keeps its whole interval
  const bool tier = (st.flags & WF_TIER_ALL) || !(st.flags & WF_DONE);
  const uint32_t rhi = st.rlo + (st.shift >= 32 ? 0xFFFFFFFFu : (1u << st.shift)) - 1u;
  float s[W_SLOTS];
  wide_load<NT>(a.scores + (long long)bh * a.cand_stride, chunk0, tid, N, a.cand_stride, s);
  int pg[W_SLOTS / 4];                            // logical page of each group of 4 slots (page lists only)
#pragma unroll
  for (int v = 0; v < W_SLOTS / 4; ++v) {
    pg[v] = 0;
    if (a.sel_pages) {
      const int pi = wide_slot<NT>(chunk0, v, tid) >> 4;
      pg[v] = a.sel_pages[(long long)bh * a.max_sel + (pi < a.max_sel ? pi : a.max_sel - 1)];
    }
  }
  uint32_t mask = 0, umask = 0;                   // bit e: slot e of this thread is kept / undecided
#pragma unroll
  for (int e = 0; e < W_SLOTS; ++e) {
    const bool valid = s[e] > -__builtin_inff();
    bool keep, und = false;
    if (a.keep_all) keep = valid;
    else {
      const uint32_t r = hp_rank_only(m, s[e]);
      const bool part = valid && r != HP_NONE;
      keep = part && (r < st.rlo || (tier && r <= rhi));
      und = part && !tier && r >= st.rlo && r <= rhi;
    }
    mask |= (keep ? 1u : 0u) << e;
    umask |= (und ? 1u : 0u) << e;
  }
  // undecided scores go onto the head's list: one atomic per wave reserves room for all its lanes
  {
    const uint32_t mine = __popc(umask);
    const uint32_t incl = tw_wave_scan_u32(mine);
    const uint32_t wtotal = __shfl(incl, 63, 64);
    if (wtotal) {                                   // wave-uniform
      uint32_t ubase = 0;
      if (lane == 63) ubase = atomicAdd(&a.ucount[(long long)bh * TW_CTR], wtotal);
      uint32_t at = __shfl(ubase, 63, 64) + incl - mine;
#pragma unroll
      for (int e = 0; e < W_SLOTS; ++e) {
        if ((umask >> e) & 1u) {
          if (at < (uint32_t)W_CAP) {
            const int slot = wide_slot<NT>(chunk0, e >> 2, tid) + (e & 3);
            const int tok = a.sel_pages ? pg[e >> 2] * TW_PAGE + (slot & 15) : slot;
            a.ulist[(long long)bh * W_CAP + at] = make_uint2(tw_float_key(s[e]), (uint32_t)tok);
          }
          ++at;
        }
      }
    }
  }
  // bitmap: the 4 bits of a group join those of the neighbouring lanes (4 lanes = one page of 16
  // slots, 8 lanes = one word of 32 slots) through DPP, then one lane stores
  uint32_t* bm = a.bitmaps + (long long)bh * a.words_stride;
#pragma unroll
  for (int v = 0; v < W_SLOTS / 4; ++v) {
    const int c = wide_slot<NT>(chunk0, v, tid);
    uint32_t x = ((mask >> (4 * v)) & 0xFu) << (4 * (lane & 7));
    x |= (uint32_t)tw_dpp_i<TW_DPP_XOR1>((int)x);
    x |= (uint32_t)tw_dpp_i<TW_DPP_XOR2>((int)x);
    if (a.sel_pages) {                            // one 16-bit half word per selected page
      const uint32_t half = (x >> (16 * ((lane >> 2) & 1))) & 0xFFFFu;
      if ((lane & 3) == 0 && (c >> 4) < count && pg[v] >= 0 && (pg[v] >> 1) < a.words_stride)   // ids outside the row: no bits, no store
        ((unsigned short*)bm)[pg[v]] = (unsigned short)half;
    } else {                                      // slots are token positions: one word per 8 lanes
      x |= (uint32_t)tw_dpp_i<TW_DPP_HALF_MIRROR>((int)x);
      if ((lane & 7) == 0 && c < N && (c >> 5) < a.words_stride) bm[c >> 5] = x;
    }
  }
  uint32_t cnt = tw_wave_scan_u32(__popc(mask));
  __shared__ uint32_t wc[16];
  if (lane == 63) wc[wave] = cnt;
  __syncthreads();
  if (tid == 0) {
    uint32_t t = 0;
    for (int w = 0; w < NT / 64; ++w) t += wc[w];
    if (t) atomicAdd(&a.kdef[(long long)bh * TW_CTR], t);
  }
}

// One workgroup per head.  The undecided scores (rank inside the interval that the passes over
// the whole row ended with) sit in registers, 4 per thread; the interval is narrowed 9 bits per
// round with a 512-bucket LDS histogram until at most 64 scores are left, and those are compared
// exactly on the scores' own bits: T = the largest key whose upper set reaches the target mass.
constexpr int WR_EPT = W_CAP / 1024;
constexpr int WR_CAP = 64;
__global__ __launch_bounds__(1024) void wide_resolve_kernel(WideArgs a) {
  const int bh = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const WideState st = a.state[bh];
  __shared__ unsigned long long histM[HP_NB];
  __shared__ uint32_t histC[HP_NB];
  __shared__ unsigned long long cand_mass[WR_CAP];
  __shared__ uint32_t cand_key[WR_CAP];
  __shared__ uint32_t red[16];
  __shared__ uint32_t sh_n, sh_T;
  const bool search = !a.keep_all && st.mk != 0 && (st.flags & WF_DONE) && !(st.flags & WF_TIER_ALL);
  uint32_t cn = 0;
  if (search) { cn = a.ucount[(long long)bh * TW_CTR]; if (cn > (uint32_t)W_CAP) cn = W_CAP; }
  const float m = tw_key_to_float(st.mk);
  uint32_t key[WR_EPT], tok[WR_EPT], rk[WR_EPT];
  float ef[WR_EPT];
#pragma unroll
  for (int e = 0; e < WR_EPT; ++e) {
    const uint32_t i = (uint32_t)(e * 1024 + tid);
    const uint2 x = a.ulist[(long long)bh * W_CAP + (i < cn ? i : 0u)];   // cn = 0: slot 0 is inside the buffer, masked
    key[e] = x.x; tok[e] = x.y;
    rk[e] = i < cn ? hp_rank(m, tw_key_to_float(x.x), &ef[e]) : HP_NONE;
  }
  if (tid == 0) sh_n = 0;
  __syncthreads();
  uint32_t T = 0xFFFFFFFFu;                         // nothing from the list unless a threshold is found
  if (cn > 0) {                                     // block-uniform
    uint32_t rlo = st.rlo, pop = cn;
    int shift = (int)st.shift;
    unsigned long long A = st.A;
    const unsigned long long target = st.target;
#pragma unroll 1
    while (pop > (uint32_t)WR_CAP && shift > 0) {
      const int nshift = shift >= 9 ? shift - 9 : 0;
      const uint32_t nb = 1u << (shift - nshift);   // buckets that cover the interval
      for (int i = tid; i < HP_NB; i += 1024) { histM[i] = 0; histC[i] = 0; }
      __syncthreads();
#pragma unroll
      for (int e = 0; e < WR_EPT; ++e) {
        if (rk[e] != HP_NONE && rk[e] >= rlo) {
          const uint32_t bk = (rk[e] - rlo) >> nshift;
          if (bk < nb) { atomicAdd(&histM[bk], hp_fix(ef[e])); atomicAdd(&histC[bk], 1u); }
        }
      }
      __syncthreads();
      unsigned long long mb[8], mine = 0;           // every wave scans on its own: lane l owns buckets 8l .. 8l+7
#pragma unroll
      for (int k = 0; k < 8; ++k) { mb[k] = histM[8 * lane + k]; mine += mb[k]; }
      const unsigned long long incl = tw_wave_scan_u64(mine);
      const unsigned long long before = A + incl - mine;
      const bool hit = before < target && before + mine >= target;
      const unsigned long long bal = __ballot(hit);
      if (bal == 0) { pop = 0xFFFFFFFFu; shift = nshift; break; }   // unreachable: the interval holds the crossing
      const int src = __ffsll((long long)bal) - 1;
      unsigned long long cum = before, asel = before;
      int bsel = 0;
#pragma unroll
      for (int k = 0; k < 8; ++k) {
        if (cum < target && cum + mb[k] >= target) { bsel = k; asel = cum; }
        cum += mb[k];
      }
      const int bucket = 8 * src + __shfl(bsel, src, 64);
      A = __shfl(asel, src, 64);
      pop = histC[bucket];
      rlo += (uint32_t)bucket << nshift;
      shift = nshift;
      __syncthreads();                              // all scans done before the histogram is cleared
    }
    const uint32_t rhi = rlo + (1u << shift) - 1u;
    const bool small = pop <= (uint32_t)WR_CAP;
    uint32_t kmin = 0xFFFFFFFFu;
#pragma unroll
    for (int e = 0; e < WR_EPT; ++e) {
      if (rk[e] != HP_NONE && rk[e] >= rlo && rk[e] <= rhi) {
        kmin = key[e] < kmin ? key[e] : kmin;
        if (small) {
          const uint32_t at = atomicAdd(&sh_n, 1u);
          if (at < (uint32_t)WR_CAP) { cand_key[at] = key[e]; cand_mass[at] = hp_fix(ef[e]); }
        }
      }
    }
    if (!small) {                                   // more than WR_CAP scores of one rank: keep them all
      kmin = ~tw_wave_max_u32(~kmin);
      if (lane == 0) red[wave] = kmin;
    }
    __syncthreads();
    if (wave == 0) {
      if (small) {
        const uint32_t n = sh_n < (uint32_t)WR_CAP ? sh_n : (uint32_t)WR_CAP;
        const uint32_t kx = lane < (int)n ? cand_key[lane] : 0u;
        unsigned long long S = 0;
#pragma unroll 4
        for (uint32_t j = 0; j < n; ++j) S += cand_key[j] >= kx ? cand_mass[j] : 0ull;
        const uint32_t best = (lane < (int)n && A + S >= target) ? kx : 0u;
        T = tw_wave_max_u32(best);
      } else {
        uint32_t r = red[0];
#pragma unroll
        for (int w = 1; w < 16; ++w) r = red[w] < r ? red[w] : r;
        T = r;
      }
      if (lane == 0) sh_T = T;
    }
    __syncthreads();
    T = sh_T;
    if (T == 0) T = 0xFFFFFFFFu;                    // unreachable (the interval holds the crossing): keep none of the list
    __syncthreads();                                // red is reused below
  }
  uint32_t add = 0;
#pragma unroll
  for (int e = 0; e < WR_EPT; ++e) {
    if (rk[e] != HP_NONE && key[e] >= T && (tok[e] >> 5) < (uint32_t)a.words_stride) {
      atomicOr(&a.bitmaps[(long long)bh * a.words_stride + (tok[e] >> 5)], 1u << (tok[e] & 31));
      add += 1;
    }
  }
  add = tw_wave_scan_u32(add);
  if (lane == 63) red[wave] = add;
  __syncthreads();
  if (tid == 0) {
    uint32_t t = a.kdef[(long long)bh * TW_CTR];
    for (int w = 0; w < 16; ++w) t += red[w];
    a.kept_count[bh] = (int32_t)t;
  }
}

struct ListArgs {
  const uint32_t* bitmaps;
  const int32_t* seq_lens;
  int32_t* count_out;         // or nullptr (count already known)
  int32_t* idx_out;
  uint32_t* status;
  int rows_per_seq, maps_per_row, max_pages, words_stride, out_stride;
  uint32_t trunc_bit;
  uint32_t* segcnt;           // [row][segs]: set bits per segment, filled by bitmap_count_kernel; nullptr = count in place
  int segs;
};

// Row r: OR of NB consecutive bitmaps (r * maps_per_row ...) -> ascending positions.  One
// workgroup per (segment of 256 words, row): its output offset is the number of bits in the
// row's earlier segments - read from the per-segment counts that bitmap_count_kernel left
// (long rows), or counted in place (rows of a few segments); it then stages its own positions
// in LDS and copies them out coalesced.  The workgroup of the last segment also writes the count.
constexpr int BL_SEG = 256;
template <int NB>
__global__ __launch_bounds__(256) void bitmap_count_kernel(ListArgs a) {
  const int row = blockIdx.y, seg = blockIdx.x, tid = threadIdx.x;
  const uint32_t* bm = a.bitmaps + (long long)row * a.maps_per_row * a.words_stride;
  const int wi = seg * BL_SEG + tid;
  uint32_t w = 0;
  if (wi < a.words_stride) {
#pragma unroll
    for (int hh = 0; hh < NB; ++hh) w |= bm[(long long)hh * a.words_stride + wi];
  }
  __shared__ uint32_t ws32[16];
  uint32_t total;
  tw_block_scan_u32(__popc(w), ws32, &total);
  if (tid == 0) a.segcnt[(long long)row * a.segs + seg] = total;
}

template <int NB>
__global__ __launch_bounds__(256) void bitmap_list_kernel(ListArgs a) {
  const int row = blockIdx.y, seg = blockIdx.x, b = row / a.rows_per_seq, tid = threadIdx.x;
  const int n = a.seq_lens[b];
  int P = n > 0 ? (n + TW_PAGE - 1) / TW_PAGE : 0;
  if (P > a.max_pages) P = a.max_pages;
  const int ntok = P * TW_PAGE < n ? P * TW_PAGE : n;
  const int nwords = (ntok + 31) >> 5;
  const int nseg = (nwords + BL_SEG - 1) / BL_SEG;
  if (seg >= nseg && !(seg == 0 && nseg == 0)) return;
  __shared__ uint32_t ws32[16];
  __shared__ int32_t stage[BL_SEG * 32];
  const uint32_t* bm = a.bitmaps + (long long)row * a.maps_per_row * a.words_stride;
  int32_t* out = a.idx_out + (long long)row * a.out_stride;
  // bits before this segment
  uint32_t before = 0;
  if (a.segcnt) {
    for (int s0 = tid; s0 < seg; s0 += 256) before += a.segcnt[(long long)row * a.segs + s0];
  } else
  for (int s0 = 0; s0 < seg; s0 += 4) {             // 4 clamped loads in flight
    uint32_t x[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const bool ok = s0 + j < seg;
      const int wi = ok ? (s0 + j) * BL_SEG + tid : 0;
      uint32_t v = 0;
#pragma unroll
      for (int hh = 0; hh < NB; ++hh) v |= bm[(long long)hh * a.words_stride + wi];
      x[j] = ok ? v : 0u;
    }
    before += __popc(x[0]) + __popc(x[1]) + __popc(x[2]) + __popc(x[3]);
  }
  const int wi = seg * BL_SEG + tid;
  uint32_t w = 0;
  if (wi < nwords) {
#pragma unroll
    for (int hh = 0; hh < NB; ++hh) w |= bm[(long long)hh * a.words_stride + wi];
  }
  uint32_t base_total, total;
  tw_block_scan_u32(before, ws32, &base_total);
  const uint32_t incl = tw_block_scan_u32(__popc(w), ws32, &total);
  uint32_t pos = incl - __popc(w);
  while (w) {
    const int bit = __ffs(w) - 1;
    w &= w - 1;
    stage[pos++] = wi * 32 + bit;
  }
  __syncthreads();
  for (uint32_t i = tid; i < total; i += 256)
    if (base_total + i < (uint32_t)a.out_stride) out[base_total + i] = stage[i];
  if (tid == 0 && seg == (nseg > 0 ? nseg - 1 : 0)) {
    uint32_t run = base_total + total;
    if (run > (uint32_t)a.out_stride) { atomicOr(a.status, a.trunc_bit); run = a.out_stride; }
    if (a.count_out) a.count_out[row] = (int32_t)run;
  }
}

template <int NB>
int launch_list(ListArgs a, int rows, uint32_t* segcnt, hipStream_t s) {
  int err = TW_OK;
  const int max_words = (a.max_pages + 1) / 2;
  int segs = (max_words + BL_SEG - 1) / BL_SEG;
  if (segs < 1) segs = 1;
  a.segs = segs;
  a.segcnt = segs > 4 ? segcnt : nullptr;           // few segments: counting the earlier ones in place is cheaper than a launch
  if (a.segcnt) {                                    // a launch of its own: close the caller's bracket, open another
    TW_LAUNCH(bitmap_count_kernel<NB>, dim3(segs, rows), dim3(256), 0, s, a);
    err = tw_prof_after(s);
    tw_prof_before(TW_K_UNION, s);
  }
  TW_LAUNCH(bitmap_list_kernel<NB>, dim3(segs, rows), dim3(256), 0, s, a);
  return err;
}

}  // namespace

// Everything after the scores have been written (and headmax filled by the scoring kernel).
// tw_prune_wide_init must have been enqueued BEFORE the scoring kernel.
int tw_prune_wide_init(const TwDims& d, const PruneWs& L, void* ws, hipStream_t s) {
  const size_t n16 = (L.state - L.headmax) / 16;
  const int nbh = d.batch * d.Hq;
  const size_t n = n16 > (size_t)nbh ? n16 : (size_t)nbh;
  tw_prof_before(TW_K_TOPP, s);
  TW_LAUNCH(wide_init_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s,
                     (uint4*)((char*)ws + L.headmax), n16, (WideState*)((char*)ws + L.state), nbh);
  return tw_prof_after(s);
}

int tw_prune_wide(const TwDims& d, const PruneWs& L, void* ws, const twilight_kv_t* kv, const int32_t* sel_pages,
                  const int32_t* sel_count, int max_sel, int cand_stride, float p, int32_t* kept_count,
                  int32_t* kept_idx, int kept_stride, int32_t* union_count, int32_t* union_idx, int union_stride,
                  uint32_t* status, hipStream_t s) {
  char* base = (char*)ws;
  WideArgs a;
  a.scores = (const float*)(base + L.scores); a.sel_pages = sel_pages; a.sel_count = sel_count; a.seq_lens = kv->seq_lens;
  a.headmax = (const uint32_t*)(base + L.headmax); a.state = (WideState*)(base + L.state);
  a.ghistM = (unsigned long long*)(base + L.ghistM); a.ghistC = (uint32_t*)(base + L.ghistC);
  a.ulist = (uint2*)(base + L.ulist);
  a.ucount = (uint32_t*)(base + L.ucount); a.kdef = (uint32_t*)(base + L.kdef);
  a.bitmaps = (uint32_t*)(base + L.bitmaps); a.kept_count = kept_count; a.status = status;
  a.Hq = d.Hq; a.max_pages = d.max_pages; a.max_sel = max_sel; a.cand_stride = cand_stride;
  a.words_stride = L.words_stride; a.keep_all = p >= 1.0f ? 1 : 0; a.p = p;
  const int nbh = d.batch * d.Hq;
  // measured at 4 x 262144 tokens x 64 heads: histogram pass 72 / 77 / 83 us with 1024 / 512 / 256 threads (fewer
  // flushes of the LDS histogram per score), emit pass 86 / 69 / 58 us (small workgroups overlap their load and
  // compute phases; at 88 registers only one 1024-thread workgroup fits a CU)
  constexpr int HIST_NT = 1024, EMIT_NT = 256;
#ifdef TW_TUNING                                 // tuning builds only: the shipped library reads no environment
  static const int emit_nt = getenv("TW_WIDE_EMIT_NT") ? atoi(getenv("TW_WIDE_EMIT_NT")) : EMIT_NT;
  static const int hist_nt = getenv("TW_WIDE_HIST_NT") ? atoi(getenv("TW_WIDE_HIST_NT")) : HIST_NT;
#else
  constexpr int emit_nt = EMIT_NT, hist_nt = HIST_NT;
#endif
  auto grid_for = [&](int nt) { return dim3((cand_stride + nt * W_SLOTS - 1) / (nt * W_SLOTS), nbh); };
  if (!a.keep_all) {
    // pass 0 locates the 1/64-logit bucket of the threshold; two 11-bit refinements at most follow
    // (a head stops as soon as <= 4096 scores are left, normally after pass 0; its later passes
    //  return at once)
    for (int pass = 0; pass < 3; ++pass) {
      tw_prof_before(TW_K_TOPP, s);
      if (hist_nt == 256)      TW_LAUNCH(wide_hist_kernel<256>, grid_for(256), dim3(256), 0, s, a);
      else if (hist_nt == 512) TW_LAUNCH(wide_hist_kernel<512>, grid_for(512), dim3(512), 0, s, a);
      else                     TW_LAUNCH(wide_hist_kernel<1024>, grid_for(1024), dim3(1024), 0, s, a);
      if (int e = tw_prof_after(s)) return e;
      tw_prof_before(TW_K_TOPP, s);
      TW_LAUNCH(wide_decide_kernel, dim3(nbh), dim3(64), 0, s, a);
      if (int e = tw_prof_after(s)) return e;
    }
  }
  tw_prof_before(TW_K_TOPP, s);
  if (emit_nt == 128)       TW_LAUNCH(wide_emit_kernel<128>, grid_for(128), dim3(128), 0, s, a);
  else if (emit_nt == 512)  TW_LAUNCH(wide_emit_kernel<512>, grid_for(512), dim3(512), 0, s, a);
  else if (emit_nt == 1024) TW_LAUNCH(wide_emit_kernel<1024>, grid_for(1024), dim3(1024), 0, s, a);
  else                      TW_LAUNCH(wide_emit_kernel<256>, grid_for(256), dim3(256), 0, s, a);
  if (int e = tw_prof_after(s)) return e;
  tw_prof_before(TW_K_TOPP, s);
  TW_LAUNCH(wide_resolve_kernel, dim3(nbh), dim3(1024), 0, s, a);
  if (int e = tw_prof_after(s)) return e;

  uint32_t* segcnt = (uint32_t*)(base + L.segcnt);
  ListArgs l;
  l.bitmaps = a.bitmaps; l.seq_lens = kv->seq_lens; l.status = status; l.max_pages = d.max_pages;
  l.words_stride = L.words_stride;
  if (kept_idx) {
    l.count_out = kept_count; l.idx_out = kept_idx; l.rows_per_seq = d.Hq; l.maps_per_row = 1; l.out_stride = kept_stride;
    l.trunc_bit = TW_STATUS_KEPT_TRUNCATED;
    tw_prof_before(TW_K_UNION, s);
    const int le = launch_list<1>(l, nbh, segcnt, s);
    if (int e = tw_prof_after(s)) return e;
    if (le) return le;
  }
  l.count_out = union_count; l.idx_out = union_idx; l.rows_per_seq = d.Hkv; l.maps_per_row = d.G; l.out_stride = union_stride;
  l.trunc_bit = TW_STATUS_UNION_TRUNCATED;
  tw_prof_before(TW_K_UNION, s);
  int le;
  switch (d.G) {
    case 1: le = launch_list<1>(l, d.batch * d.Hkv, segcnt, s); break;
    case 2: le = launch_list<2>(l, d.batch * d.Hkv, segcnt, s); break;
    case 4: le = launch_list<4>(l, d.batch * d.Hkv, segcnt, s); break;
    default: le = launch_list<8>(l, d.batch * d.Hkv, segcnt, s); break;
  }
  if (int e = tw_prof_after(s)) return e;
  return le;
}
