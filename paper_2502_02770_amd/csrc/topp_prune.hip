// Stage 2: the Twilight pruner (paper: Section 4.2, Algorithm 1,
// Definition 3.3, Appendix B.1 and B.2).
//
// int4_score       estimated logits from the quantised K copy.  One wave = one
//                  page per step: 64 lanes x 16 B = the page's 1 KiB of codes,
//                  lane = (token, group of 32 dims); 8 integer dot4 per lane
//                  and head, scale/zero applied per group, quad DPP sum over
//                  the 4 groups.  Templated on the code width (2 / 4 / 8 bits).
// int4_score_mfma  the same scores on the matrix cores, used when every page
//                  is a candidate and 4 or 8 query heads share each page.
// topp_head        per (sequence, query head), scores in registers: max, then
//                  a mass histogram over the fixed-point distance to the max
//                  logit narrows the threshold 9 bits per pass (masses in
//                  64-bit fixed point, so sums do not depend on the order of
//                  the atomics), finished by an exact resolve on the scores'
//                  own bit patterns inside one wave.  Kept tokens go to a
//                  bitmap; the last head of a KV group to finish ORs the
//                  group's bitmaps into the sorted union list.
// Rows too long for registers take the multi-workgroup path in topp_wide.hip.
#include <stdlib.h>
#include "topp_common.h"
#include "select_body.h"

namespace {

constexpr float kInv127 = 0x1.020408p-7f;    // fp32(1/127)
constexpr float kRsqrtD = 0x1.6a09e6p-4f;    // fp32(1/sqrt(128))

// ------------------------------------------------------------------ int4_score
struct ScoreArgs {
  const uint16_t* q;          // bf16 [b][Hq][128]
  const int32_t* sel_pages;   // [b][Hq][max_sel] or nullptr (all pages)
  const int32_t* sel_count;
  const int32_t* page_table;
  const int32_t* seq_lens;
  const uint4* kq_pool;       // 64 uint4 per (page, head)
  const uint32_t* kq_meta;    // 64 words per (page, head)
  float* scores;              // [b][Hq][cand_stride]
  int32_t* dots;              // [b][Hq][cand_stride][4] or nullptr
  uint32_t* arrive;           // [b][Hkv] arrival counters of the top-p kernel that follows, or nullptr
  uint32_t* headmax;          // [b][Hq][HM_SLOTS] keys whose maximum is the head's largest score (atomicMax), or nullptr
  const uint32_t* chmask;     // [Hkv][4] channels of the query that take part (bit d % 32 of word d / 32), or nullptr = all
  int Hq, Hkv, max_pages, max_sel, cand_stride, pw;   // pw: pages per wave (<= 64)
  int rotate;                 // list mode with a grid a multiple of 8 wide: chunk = (column - group % 8) mod width
  long long pool_pages;
};

// q of NH consecutive heads -> int8 (symmetric per head: sq = max|q| * (1/127), round half even),
// 4 values per word, and c = sq / sqrt(128) per head.  Called by all threads of the block (>= 128).
// chmask: 4 words of the KV head's channel set, or nullptr - channels outside it get the int8 value 0 (the scale sq
// is that of the whole query), which restricts the estimate to the set (channel-sparse token selector).
template <int NH>
__device__ __forceinline__ void tw_quantize_q(const uint16_t* q, int (*qi_s)[32], float* red, float* c_s,
                                              const uint32_t* chmask = nullptr) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
#pragma unroll 1
  for (int h = 0; h < NH; ++h) {
    float v = 0.f;
    if (tid < 128) v = __uint_as_float((uint32_t)q[h * 128 + tid] << 16);
    float av = fabsf(v);
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) av = fmaxf(av, __shfl_xor(av, o, 64));
    if (lane == 0 && wave < 2) red[wave] = av;     // the 128 values sit in waves 0 and 1
    __syncthreads();
    const float amax = fmaxf(red[0], red[1]);
    const float sq = __fmul_rn(amax, kInv127);
    if (tid < 128) {
      int qi = 0;
      if (sq > 0.f) {
        float t = rintf(__fdiv_rn(v, sq));
        t = fminf(fmaxf(t, -127.f), 127.f);
        qi = (int)t;
      }
      if (chmask && !((chmask[tid >> 5] >> (tid & 31)) & 1u)) qi = 0;
      ((int8_t*)qi_s[h])[tid] = (int8_t)qi;
    }
    if (tid == 0) c_s[h] = __fmul_rn(sq, kRsqrtD);
    __syncthreads();
  }
}

// The same for one head whose 128 values the threads 0..127 already hold (v; others pass 0).
__device__ __forceinline__ void tw_quantize_q1(float v, int (*qi_s)[32], float* red, float* c_s) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  float av = fabsf(v);
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) av = fmaxf(av, __shfl_xor(av, o, 64));
  if (lane == 0 && wave < 2) red[wave] = av;
  __syncthreads();
  const float sq = __fmul_rn(fmaxf(red[0], red[1]), kInv127);
  if (tid < 128) {
    int qi = 0;
    if (sq > 0.f) {
      float t = rintf(__fdiv_rn(v, sq));
      t = fminf(fmaxf(t, -127.f), 127.f);
      qi = (int)t;
    }
    ((int8_t*)qi_s[0])[tid] = (int8_t)qi;
  }
  if (tid == 0) c_s[0] = __fmul_rn(sq, kRsqrtD);
  __syncthreads();
}

// One lane's group of 32 codes of slot (token, group) `idx` of the pool, as 8 dot4 operands
// (4 dims each, in the order of the query words); 8-bit codes come out as code - 128.
// STREAM: the codes are read once (every page a candidate, all heads of the group in one workgroup) and loaded
// non-temporally; with per-head page lists they stay cached for the other heads of the group.
template <int BITS, bool STREAM = false>
__device__ __forceinline__ void tw_load_codes(const uint4* kq_pool, long long idx, int (&u)[8]) {
  if (BITS == 4) {
    const uint4 nib = STREAM ? tw_ld_stream(kq_pool + idx) : kq_pool[idx];
    u[0] = nib.x & 0x0F0F0F0F; u[1] = (nib.x >> 4) & 0x0F0F0F0F;
    u[2] = nib.y & 0x0F0F0F0F; u[3] = (nib.y >> 4) & 0x0F0F0F0F;
    u[4] = nib.z & 0x0F0F0F0F; u[5] = (nib.z >> 4) & 0x0F0F0F0F;
    u[6] = nib.w & 0x0F0F0F0F; u[7] = (nib.w >> 4) & 0x0F0F0F0F;
  } else if (BITS == 2) {
    const uint2 cr = ((const uint2*)kq_pool)[idx];
    u[0] = cr.x & 0x03030303; u[1] = (cr.x >> 2) & 0x03030303; u[2] = (cr.x >> 4) & 0x03030303; u[3] = (cr.x >> 6) & 0x03030303;
    u[4] = cr.y & 0x03030303; u[5] = (cr.y >> 2) & 0x03030303; u[6] = (cr.y >> 4) & 0x03030303; u[7] = (cr.y >> 6) & 0x03030303;
  } else {
    const uint4 c0 = kq_pool[idx * 2], c1 = kq_pool[idx * 2 + 1];
    u[0] = c0.x ^ 0x80808080; u[1] = c0.y ^ 0x80808080; u[2] = c0.z ^ 0x80808080; u[3] = c0.w ^ 0x80808080;
    u[4] = c1.x ^ 0x80808080; u[5] = c1.y ^ 0x80808080; u[6] = c1.z ^ 0x80808080; u[7] = c1.w ^ 0x80808080;
  }
}
// The same in two steps, so that a kernel can ask for several slots' codes before it unpacks the first.
template <int BITS, bool STREAM = false>
__device__ __forceinline__ void tw_load_raw(const uint4* kq_pool, long long idx, uint4 (&r)[BITS == 8 ? 2 : 1]) {
  if (BITS == 4) r[0] = STREAM ? tw_ld_stream(kq_pool + idx) : kq_pool[idx];
  else if (BITS == 2) { const uint2 c = ((const uint2*)kq_pool)[idx]; r[0] = make_uint4(c.x, c.y, 0u, 0u); }
  else { r[0] = kq_pool[idx * 2]; r[BITS == 8 ? 1 : 0] = kq_pool[idx * 2 + 1]; }
}
template <int BITS>
__device__ __forceinline__ void tw_unpack_codes(const uint4 (&r)[BITS == 8 ? 2 : 1], int (&u)[8]) {
  if (BITS == 4) {
    u[0] = r[0].x & 0x0F0F0F0F; u[1] = (r[0].x >> 4) & 0x0F0F0F0F;
    u[2] = r[0].y & 0x0F0F0F0F; u[3] = (r[0].y >> 4) & 0x0F0F0F0F;
    u[4] = r[0].z & 0x0F0F0F0F; u[5] = (r[0].z >> 4) & 0x0F0F0F0F;
    u[6] = r[0].w & 0x0F0F0F0F; u[7] = (r[0].w >> 4) & 0x0F0F0F0F;
  } else if (BITS == 2) {
    u[0] = r[0].x & 0x03030303; u[1] = (r[0].x >> 2) & 0x03030303; u[2] = (r[0].x >> 4) & 0x03030303; u[3] = (r[0].x >> 6) & 0x03030303;
    u[4] = r[0].y & 0x03030303; u[5] = (r[0].y >> 2) & 0x03030303; u[6] = (r[0].y >> 4) & 0x03030303; u[7] = (r[0].y >> 6) & 0x03030303;
  } else {
    constexpr int H = BITS == 8 ? 1 : 0;
    u[0] = r[0].x ^ 0x80808080; u[1] = r[0].y ^ 0x80808080; u[2] = r[0].z ^ 0x80808080; u[3] = r[0].w ^ 0x80808080;
    u[4] = r[H].x ^ 0x80808080; u[5] = r[H].y ^ 0x80808080; u[6] = r[H].z ^ 0x80808080; u[7] = r[H].w ^ 0x80808080;
  }
}
// I = sum over the group's 32 dims of q * code (i0 = 128 * sum q for 8-bit codes, else 0)
__device__ __forceinline__ int tw_group_dot(const int (&qw)[8], const int (&u)[8], int i0) {
  int I = __builtin_amdgcn_sdot4(qw[0], u[0], i0, false);
  I = __builtin_amdgcn_sdot4(qw[1], u[1], I, false);
  I = __builtin_amdgcn_sdot4(qw[2], u[2], I, false);
  I = __builtin_amdgcn_sdot4(qw[3], u[3], I, false);
  I = __builtin_amdgcn_sdot4(qw[4], u[4], I, false);
  I = __builtin_amdgcn_sdot4(qw[5], u[5], I, false);
  I = __builtin_amdgcn_sdot4(qw[6], u[6], I, false);
  I = __builtin_amdgcn_sdot4(qw[7], u[7], I, false);
  return I;
}
// the group's term of the score: fl(scale * I) + fl(zero * sum q), summed over the 4 groups of the
// token (the 4 lanes of a quad) in the fixed order (T0 + T1) + (T2 + T3)
__device__ __forceinline__ float tw_token_sum(uint32_t meta, int I, float qsf) {
  const float sc = __half2float(__ushort_as_half((unsigned short)(meta & 0xFFFFu)));
  const float ze = __half2float(__ushort_as_half((unsigned short)(meta >> 16)));
  return tw_quad_sum(__fadd_rn(__fmul_rn(sc, (float)I), __fmul_rn(ze, qsf)));
}

// NH = heads scored per loaded page: 1 with per-head page lists, G when every
// page is a candidate (the G heads of a KV head then share each load).
template <int NH, bool FULL, bool DOTS, int UNR, int BITS = 4>
__global__ __launch_bounds__(256) void int4_score_kernel(ScoreArgs a) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  int b, g, h0;
  if (FULL) { b = blockIdx.y / a.Hkv; g = blockIdx.y % a.Hkv; h0 = g * NH; }
  else      { b = blockIdx.y / a.Hq;  h0 = blockIdx.y % a.Hq; g = h0 / (a.Hq / a.Hkv); }
  const int n = a.seq_lens[b];
  int P = n > 0 ? (n + TW_PAGE - 1) / TW_PAGE : 0;
  if (P > a.max_pages) P = a.max_pages;
  int count = P;
  if (!FULL) { count = a.sel_count[b * a.Hq + h0]; if (count > a.max_sel) count = a.max_sel; }
  // A workgroup takes the chunks of 4 * pw pages number blockIdx.x, blockIdx.x + gridDim.x, ... of its row
  // (one chunk each when the grid covers the row bound; fewer, looping workgroups for batches of many heads,
  // whose lists are often far shorter than the bound).
  // Workgroups go to the 8 XCDs round robin in dispatch order, so with a grid a multiple of 8 wide column x runs on XCD x % 8
  // and the heads of a KV head, which select largely the same pages, find each other's pages in that XCD's
  // L2.  Rotating the chunks by the group's number keeps that and spreads the first chunks of short lists
  // over all XCDs.
  const int col = (!FULL && a.rotate) ? (int)((blockIdx.x + gridDim.x - ((unsigned)(b * a.Hkv + g) & 7u)) % gridDim.x) : (int)blockIdx.x;
  int wg_first = col * 4 * a.pw;
  if (a.arrive && blockIdx.x == 0 && tid == 0) a.arrive[(b * a.Hkv + g) * TW_CTR] = 0;
  if (wg_first >= count) return;

  // ---- this wave's pages: lane k holds the k-th one (logical id, pool id).  The first chunk's are
  //      issued before the query is quantised, so that the two dependent loads overlap that prologue.
  int first = wg_first + wave * a.pw;
  int my_lp = -1, my_pool = -1;
  if (lane < a.pw && first + lane < count) {
    my_lp = FULL ? first + lane : a.sel_pages[((long long)(b * a.Hq + h0)) * a.max_sel + first + lane];
    if (my_lp >= 0 && my_lp < P) {
      const int pp = a.page_table[(long long)b * a.max_pages + my_lp];
      if (pp >= 0 && pp < a.pool_pages) my_pool = pp;
    }
  }
  int npages = count - first;
  if (npages > a.pw) npages = a.pw;

  // ---- quantise q of the NH heads to int8 (symmetric, per head)
  __shared__ int qi_s[NH][32];
  __shared__ float red[4];
  __shared__ float c_s[NH];
  tw_quantize_q<NH>(a.q + ((long long)(b * a.Hq + h0)) * 128, qi_s, red, c_s, a.chmask ? a.chmask + g * 4 : nullptr);
  const int j = lane & 3;                       // this lane's group of 32 dims
  int qw[NH][8], qs128[NH];
  float qsf[NH], cc[NH];
#pragma unroll
  for (int h = 0; h < NH; ++h) {
    int qs = 0;
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      qw[h][k] = qi_s[h][8 * j + k];
      qs = __builtin_amdgcn_sdot4(qw[h][k], 0x01010101, qs, false);
    }
    qsf[h] = (float)qs;
    qs128[h] = BITS == 8 ? 128 * qs : 0;        // 8-bit codes enter the signed dot4 as code - 128
    cc[h] = c_s[h];
  }

  float hm[NH];
#pragma unroll
  for (int h = 0; h < NH; ++h) hm[h] = -__builtin_inff();
#pragma unroll 1
  for (;;) {
#pragma unroll 1
  for (int k0 = 0; k0 < npages; k0 += UNR) {
   // UNR pages per round: first all their loads (unconditional: an unmapped page or one past the wave's last reads
   // pool page 0 and is masked below), so that they are in flight together, then the arithmetic
   uint4 raw[UNR][BITS == 8 ? 2 : 1];
   uint32_t metas[UNR];
   int lps[UNR], pools[UNR];
#pragma unroll
   for (int kk = 0; kk < UNR; ++kk) {
    const int k = k0 + kk;                     // wave-uniform
    lps[kk] = __builtin_amdgcn_readlane(my_lp, k & 63);
    const int pl = __builtin_amdgcn_readlane(my_pool, k & 63);
    pools[kk] = k < npages ? pl : -1;
    const long long blk = ((long long)(pools[kk] >= 0 ? pools[kk] : 0) * a.Hkv + g) * 64;
    tw_load_raw<BITS, FULL>(a.kq_pool, blk + lane, raw[kk]);
    metas[kk] = FULL ? __builtin_nontemporal_load(a.kq_meta + blk + lane) : a.kq_meta[blk + lane];
   }
#pragma unroll
   for (int kk = 0; kk < UNR; ++kk) {
    const int k = k0 + kk;
    const int lp = lps[kk], pool = pools[kk];
    int u[8];
    tw_unpack_codes<BITS>(raw[kk], u);
    const uint32_t meta = metas[kk];
    const int tok = lp * TW_PAGE + (lane >> 2);
    const bool valid = pool >= 0 && tok < n;
    const long long slot = (long long)(first + k) * TW_PAGE + (lane >> 2);
#pragma unroll
    for (int h = 0; h < NH; ++h) {
      const int I = tw_group_dot(qw[h], u, qs128[h]);
      const float T = tw_token_sum(meta, I, qsf[h]);
      const float s = valid ? __fmul_rn(T, cc[h]) : -__builtin_inff();
      if (k < npages) hm[h] = fmaxf(hm[h], s);
      const long long row = ((long long)(b * a.Hq + h0 + h)) * a.cand_stride;
      if (k < npages) {
        if (j == 0) a.scores[row + slot] = s;
        if (DOTS) a.dots[(row + slot) * 4 + j] = valid ? I : 0;
      }
    }
   }
  }
  // ---- next chunk of this workgroup, if any (block-uniform)
  wg_first += gridDim.x * 4 * a.pw;
  if (wg_first >= count) break;
  first = wg_first + wave * a.pw;
  my_lp = -1; my_pool = -1;
  if (lane < a.pw && first + lane < count) {
    my_lp = FULL ? first + lane : a.sel_pages[((long long)(b * a.Hq + h0)) * a.max_sel + first + lane];
    if (my_lp >= 0 && my_lp < P) {
      const int pp = a.page_table[(long long)b * a.max_pages + my_lp];
      if (pp >= 0 && pp < a.pool_pages) my_pool = pp;
    }
  }
  npages = count - first;
  if (npages > a.pw) npages = a.pw;
  }
  if (a.headmax) {
    // one atomic per head and workgroup: waves reduce through LDS first
    __shared__ float hm_s[4][NH];
#pragma unroll
    for (int h = 0; h < NH; ++h) {
      const float mx = tw_wave_max_f(hm[h]);
      if (lane == 0) hm_s[wave][h] = mx;
    }
    __syncthreads();
    if (tid < NH) {
      const float mx = fmaxf(fmaxf(hm_s[0][tid], hm_s[1][tid]), fmaxf(hm_s[2][tid], hm_s[3][tid]));
      if (mx > -__builtin_inff())
        atomicMax(a.headmax + ((long long)(b * a.Hq + h0 + tid) * HM_SLOTS + (blockIdx.x & (HM_SLOTS - 1))) * TW_CTR, tw_float_key(mx));
    }
  }
}

// ------------------------------------------------------------------ int4_score over token lists
// The candidates of a head are token positions handed over by any token-level selector
// (Section 4.1).  A quad of lanes owns one candidate (lane & 3 = group of 32 dims): 16 bytes of
// codes and the group's (scale, zero) per lane, gathered from the token's slot in its page; a
// workgroup covers 256 consecutive candidate slots, 64 per step, all steps' loads in flight
// together.  Same integers and fp32 operations as the page-list kernel: bit-identical scores.
template <bool DOTS, int BITS>
__global__ __launch_bounds__(256) void int4_score_tokens_kernel(ScoreArgs a) {
  constexpr int IT = 4;
  const int tid = threadIdx.x, j = tid & 3;
  const int b = blockIdx.y / a.Hq, h0 = blockIdx.y % a.Hq, g = h0 / (a.Hq / a.Hkv);
  const int n = a.seq_lens[b];
  const int ntok = n < a.max_pages * TW_PAGE ? n : a.max_pages * TW_PAGE;
  int count = a.sel_count[b * a.Hq + h0];
  if (count > a.max_sel) count = a.max_sel;
  // chunk columns as in the page-list kernel: a grid a multiple of 8 wide is rotated by the KV group's number
  const int col = a.rotate ? (int)((blockIdx.x + gridDim.x - ((unsigned)(b * a.Hkv + g) & 7u)) % gridDim.x) : (int)blockIdx.x;
  int wg_first = col * 64 * IT;
  if (a.arrive && blockIdx.x == 0 && tid == 0) a.arrive[(b * a.Hkv + g) * TW_CTR] = 0;
  if (wg_first >= count) return;

  // token -> pool slot of every step first, so that the dependent loads overlap the query prologue
  const long long row = ((long long)(b * a.Hq + h0)) * a.cand_stride;
  long long slot4[IT];                              // (token slot in the pool) * 4 + group, or -1
  auto translate = [&]() {
#pragma unroll
    for (int it = 0; it < IT; ++it) {
      const int c = wg_first + it * 64 + (tid >> 2);
      const int tok = c < count ? a.sel_pages[row + c] : -1;
      slot4[it] = -1;
      if (tok >= 0 && tok < ntok) {
        const int pp = a.page_table[(long long)b * a.max_pages + (tok >> 4)];
        if (pp >= 0 && pp < a.pool_pages) slot4[it] = ((((long long)pp * a.Hkv + g) * TW_PAGE + (tok & 15)) << 2) + j;
      }
    }
  };
  translate();

  __shared__ int qi_s[1][32];
  __shared__ float red[4];
  __shared__ float c_s[1];
  tw_quantize_q<1>(a.q + ((long long)(b * a.Hq + h0)) * 128, qi_s, red, c_s);
  int qw[8], qs = 0;
#pragma unroll
  for (int k = 0; k < 8; ++k) {
    qw[k] = qi_s[0][8 * j + k];
    qs = __builtin_amdgcn_sdot4(qw[k], 0x01010101, qs, false);
  }
  const float qsf = (float)qs, cc = c_s[0];
  const int qs128 = BITS == 8 ? 128 * qs : 0;

#pragma unroll 1
  for (;;) {
    int u[IT][8];
    uint32_t meta[IT];
#pragma unroll
    for (int it = 0; it < IT; ++it) {               // unconditional loads (an invalid candidate reads slot 0, masked below)
      const long long idx = slot4[it] >= 0 ? slot4[it] : (long long)j;
      tw_load_codes<BITS>(a.kq_pool, idx, u[it]);
      meta[it] = a.kq_meta[idx];
    }
#pragma unroll
    for (int it = 0; it < IT; ++it) {
      const int c = wg_first + it * 64 + (tid >> 2);
      const bool valid = slot4[it] >= 0;
      const int I = tw_group_dot(qw, u[it], qs128);
      const float T = tw_token_sum(meta[it], I, qsf);   // all four lanes of the quad take part
      const float sc = valid ? __fmul_rn(T, cc) : -__builtin_inff();
      if (c < count) {
        if (j == 0) a.scores[row + c] = sc;
        if (DOTS) a.dots[(row + c) * 4 + j] = valid ? I : 0;
      }
    }
    wg_first += gridDim.x * 64 * IT;                // next chunk of this workgroup, if any (block-uniform)
    if (wg_first >= count) break;
    translate();
  }
}

// ------------------------------------------------------------------ int4_score on the matrix cores
// Every page a candidate and 4 or 8 query heads per KV head: per page the scores are a small dense
// contraction, [heads x 128 dims] . [128 dims x 16 tokens], which on the vector ALU costs 8 dot4
// per lane and head and 64 registers of query words (8 heads: 130 VGPRs, 3 waves per SIMD, too few
// pages in flight to keep HBM busy).  Here v_mfma_i32_16x16x32_i8 does the integer part.  The four
// groups of 32 dims have their own (scale, zero), so their dot products must stay apart: row
// 4*h + j of the A operand carries head h's query words of group j and zeros elsewhere, and lane
// (k-block j', token t) supplies group j' of token t as B; four MFMAs (one per 8-dim word of the
// groups) accumulate I_j[h][t].  The result lands with lane (h, t) holding I_0..I_3: scale/zero,
// the fixed-order sum and the store need no cross-lane step.  Same integers and the same fp32
// operations as the vector kernel, so the scores are bit-identical.
typedef int tw_i32x4 __attribute__((ext_vector_type(4)));

template <int NHG, bool DOTS, int UNR>           // NHG groups of 4 heads
__global__ __launch_bounds__(256) void int4_score_mfma_kernel(ScoreArgs a) {
  constexpr int NH = 4 * NHG;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int b = blockIdx.y / a.Hkv, g = blockIdx.y % a.Hkv, h0 = g * NH;
  const int n = a.seq_lens[b];
  int P = n > 0 ? (n + TW_PAGE - 1) / TW_PAGE : 0;
  if (P > a.max_pages) P = a.max_pages;
  const int count = P;
  const int wg_first = blockIdx.x * 4 * a.pw;
  if (a.arrive && blockIdx.x == 0 && tid == 0) a.arrive[(b * a.Hkv + g) * TW_CTR] = 0;
  if (wg_first >= count) return;

  // ---- this wave's pages: lane k holds the k-th one (logical id, pool id)
  const int first = wg_first + wave * a.pw;
  int my_lp = -1, my_pool = -1;
  if (lane < a.pw && first + lane < count) {
    my_lp = first + lane;
    const int pp = a.page_table[(long long)b * a.max_pages + my_lp];
    if (pp >= 0 && pp < a.pool_pages) my_pool = pp;
  }
  int npages = count - first;
  if (npages > a.pw) npages = a.pw;

  __shared__ int qi_s[NH][32];
  __shared__ float red[4];
  __shared__ float c_s[NH];
  tw_quantize_q<NH>(a.q + ((long long)(b * a.Hq + h0)) * 128, qi_s, red, c_s, a.chmask ? a.chmask + g * 4 : nullptr);

  const int kb = lane >> 4, t = lane & 15;       // B operand / result: k-block (= group of dims) or head, token
  // A operand: row m = lane & 15 = 4 * head + group; this lane's k-block only meets its own group
  long aw[NHG][4];
  {
    const int hl = t >> 2, j = t & 3;
#pragma unroll
    for (int hg = 0; hg < NHG; ++hg)
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        uint32_t lo = (uint32_t)qi_s[hg * 4 + hl][8 * j + 2 * w], hi = (uint32_t)qi_s[hg * 4 + hl][8 * j + 2 * w + 1];
        if (kb != j) { lo = 0; hi = 0; }
        aw[hg][w] = (long)(((unsigned long long)hi << 32) | lo);
      }
  }
  // result side: this lane's head is kb (+ 4 per head group); sums of its query words per group
  float qsf[NHG][4], cc[NHG];
#pragma unroll
  for (int hg = 0; hg < NHG; ++hg) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      int qs = 0;
#pragma unroll
      for (int k = 0; k < 8; ++k) qs = __builtin_amdgcn_sdot4(qi_s[hg * 4 + kb][8 * j + k], 0x01010101, qs, false);
      qsf[hg][j] = (float)qs;
    }
    cc[hg] = c_s[hg * 4 + kb];
  }

  float hm[NHG];
#pragma unroll
  for (int hg = 0; hg < NHG; ++hg) hm[hg] = -__builtin_inff();
#pragma unroll 1
  for (int k0 = 0; k0 < npages; k0 += UNR) {
    uint4 nib[UNR], mt[UNR];
    int lpv[UNR];
    bool okv[UNR];
#pragma unroll
    for (int kk = 0; kk < UNR; ++kk) {           // unconditional loads (an absent page reads pool page 0, masked below)
      const int k = k0 + kk;
      lpv[kk] = __builtin_amdgcn_readlane(my_lp, k & 63);
      const int pool = k < npages ? __builtin_amdgcn_readlane(my_pool, k & 63) : -1;
      okv[kk] = pool >= 0;
      const long long blk = ((long long)(pool >= 0 ? pool : 0) * a.Hkv + g) * 64;
      // every page is read once here (all heads of the group in this workgroup): non-temporal loads
      nib[kk] = tw_ld_stream(a.kq_pool + blk + t * 4 + kb);                // group kb of token t: 32 codes
      mt[kk] = tw_ld_stream((const uint4*)a.kq_meta + (blk >> 2) + t);     // token t: 4 x (scale | zero << 16)
    }
#pragma unroll
    for (int kk = 0; kk < UNR; ++kk) {
      const int k = k0 + kk;
      if (k < npages) {                          // wave-uniform
        const uint32_t wv[4] = {nib[kk].x, nib[kk].y, nib[kk].z, nib[kk].w};
        long bw[4];
#pragma unroll
        for (int w = 0; w < 4; ++w)
          bw[w] = (long)(((unsigned long long)((wv[w] >> 4) & 0x0F0F0F0Fu) << 32) | (wv[w] & 0x0F0F0F0Fu));
        const uint32_t mv[4] = {mt[kk].x, mt[kk].y, mt[kk].z, mt[kk].w};
        const int tok = lpv[kk] * TW_PAGE + t;
        const bool valid = okv[kk] && tok < n;
        const long long slot = (long long)(first + k) * TW_PAGE + t;
#pragma unroll
        for (int hg = 0; hg < NHG; ++hg) {
          tw_i32x4 c = {0, 0, 0, 0};
#pragma unroll
          for (int w = 0; w < 4; ++w) c = __builtin_amdgcn_mfma_i32_16x16x32_i8(aw[hg][w], bw[w], c, 0, 0, 0);
          float T[4];
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            const float sc = __half2float(__ushort_as_half((unsigned short)(mv[j] & 0xFFFFu)));
            const float ze = __half2float(__ushort_as_half((unsigned short)(mv[j] >> 16)));
            T[j] = __fadd_rn(__fmul_rn(sc, (float)c[j]), __fmul_rn(ze, qsf[hg][j]));
          }
          const float ssum = __fadd_rn(__fadd_rn(T[0], T[1]), __fadd_rn(T[2], T[3]));
          const float s = valid ? __fmul_rn(ssum, cc[hg]) : -__builtin_inff();
          hm[hg] = fmaxf(hm[hg], s);
          const long long row = ((long long)(b * a.Hq + h0 + hg * 4 + kb)) * a.cand_stride;
          a.scores[row + slot] = s;
          if (DOTS) ((tw_i32x4*)a.dots)[row + slot] = valid ? c : tw_i32x4{0, 0, 0, 0};
        }
      }
    }
  }
  if (a.headmax) {
    // one atomic per head and workgroup: 16-lane rows (one head each), then the waves through LDS
    __shared__ float hm_s[4][NH];
#pragma unroll
    for (int hg = 0; hg < NHG; ++hg) {
      float mx = hm[hg];
      mx = fmaxf(mx, tw_dpp_f<TW_DPP_XOR1>(mx));
      mx = fmaxf(mx, tw_dpp_f<TW_DPP_XOR2>(mx));
      mx = fmaxf(mx, tw_dpp_f<TW_DPP_HALF_MIRROR>(mx));
      mx = fmaxf(mx, tw_dpp_f<TW_DPP_MIRROR>(mx));
      if (t == 0) hm_s[wave][hg * 4 + kb] = mx;
    }
    __syncthreads();
    if (tid < NH) {
      const float mx = fmaxf(fmaxf(hm_s[0][tid], hm_s[1][tid]), fmaxf(hm_s[2][tid], hm_s[3][tid]));
      if (mx > -__builtin_inff())
        atomicMax(a.headmax + ((long long)(b * a.Hq + h0 + tid) * HM_SLOTS + (blockIdx.x & (HM_SLOTS - 1))) * TW_CTR, tw_float_key(mx));
    }
  }
}

// ------------------------------------------------------------------ top-p per head, scores in registers
// One workgroup (1024 threads, or 512 for the short rows of a split launch) per
// (sequence, query head); thread t owns the contiguous candidate slots
// [t*EPT, (t+1)*EPT).  Rank (fixed-point distance to the max logit) and softmax
// numerator of every score are computed once and stay in registers.  Pass 0
// buckets the ranks within 8 logits of the max at 1/64 logit and only sums up
// everything further down (no atomics); the crossing bucket is narrowed 9 bits
// per pass until at most HP_CAP scores remain, which are resolved exactly on the
// score's own bits.  Every wave scans the histogram on its own, so a pass costs
// one barrier.  The kept tokens are written as a bitmap over token positions;
// the last head of a KV group to arrive turns the group's bitmaps into the
// sorted union.
struct HeadArgs {
  const float* scores;
  const int32_t* sel_pages;
  const int32_t* sel_count;
  const int32_t* seq_lens;
  int32_t* kept_count;
  int32_t* kept_idx;          // or nullptr
  uint32_t* bitmaps;          // [b][Hq][words_stride]
  uint32_t* arrive;           // [b][Hkv] arrival counters, zero on entry
  int32_t* union_count;
  int32_t* union_idx;
  uint32_t* status;
  int Hq, Hkv, max_pages, max_sel, cand_stride, kept_stride, words_stride, union_stride;
  int n_above, n_upto;        // this launch takes the heads with n_above < candidates <= n_upto
  float p;
  // scoring inside the kernel (FUSE): the query, the quantised copy of K and the page table
  const uint16_t* q;
  const int32_t* page_table;
  const uint4* kq_pool;
  const uint32_t* kq_meta;
  long long pool_pages;
  int remap;                  // FUSE: workgroup -> head mapping that keeps the heads of a KV head on one XCD
  // page selection inside the kernel as well (FUSE == 2): the bounds of all pages and the budgets; the lists go
  // to sel_pages_w / sel_count_w
  const float* bounds;        // [b][Hq][max_pages]
  const int32_t* budget;      // [b] tokens
  int32_t* sel_pages_w;
  int32_t* sel_count_w;
};

constexpr int HP_CAP = 64;                    // exact resolve handles up to this many scores
constexpr int HP_BITMAP_WORDS = 6144;         // 196608 tokens
constexpr int HP_USTAGE = 4096;               // union lists up to this length leave through LDS

// TOK: the candidates are token positions (sel_pages = the token lists, max_sel = their row length,
// sel_count in tokens) instead of pages of 16 slots.
// FUSE >= 1: the estimated scores are computed here, from the head's page list, instead of being read from the row a
// scoring launch wrote: the workgroup's waves share the list (one page of 64 (token, group) lanes per wave and step,
// the arithmetic of int4_score_kernel), the scores cross to their owner threads through LDS.
// FUSE == 2: the page list too is made here, from the bounds of all pages (the selection of page_select_lds_kernel).
template <int NT, int EPT, int G, bool TOK = false, int FUSE = 0>
__global__ __launch_bounds__(NT, NT == 512 ? 6 : 1) void topp_head_kernel(HeadArgs a) {
  constexpr int NW = NT / 64;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  int b_ = blockIdx.y, h_ = blockIdx.x;
  if (FUSE && a.remap) {
    // Workgroups go to the 8 XCDs round robin in dispatch order.  The G heads of a KV head select largely the
    // same pages: they take G consecutive workgroups of one XCD, so that each finds the others' pages in its L2.
    const unsigned L = blockIdx.y * gridDim.x + blockIdx.x, xcd = L & 7u, r = L >> 3;
    const unsigned grp = (r / G) * 8u + xcd;             // (sequence, KV head), batch * Hkv a multiple of 8
    b_ = (int)(grp / (unsigned)a.Hkv);
    h_ = (int)(grp % (unsigned)a.Hkv) * G + (int)(r % G);
  }
  const int b = b_, h = h_;
  const int bh = b * a.Hq + h;
  // FUSE == 2: everything the page selection reads is asked for here, before the sequence's length is known (any
  // entry of the head's row of bounds and of the sequence's page-table row may be read): the bounds of the pages
  // j * NT + tid and the page-table entries of the pages tid * SEL_E + e, which this thread will list
  // (1024-thread workgroups, 4 entries each; the 512-thread form, short of registers, asks when it knows the length)
  constexpr int SEL_E = 4096 / NT;
  constexpr bool SEL_EARLY = FUSE == 2 && NT >= 1024;
  const int n = a.seq_lens[b];
  const int budget_b = FUSE == 2 ? a.budget[b] : 0;
  float sel_pre[SEL_EARLY ? SEL_E : 1];
  int32_t sel_pt[FUSE == 2 ? SEL_E : 1];
  // (when the heads are split over two launches by list length, half the workgroups of each return at once: those
  //  must not leave with loads in flight, so the loads then follow the test)
  const bool all_heads = a.n_above < 0 && a.n_upto >= a.cand_stride;
  auto ask_selection = [&]() {
#pragma unroll
    for (int j = 0; j < SEL_E; ++j) {
      const int i = j * NT + tid, e = tid * SEL_E + j;
      sel_pre[SEL_EARLY ? j : 0] = a.bounds[(long long)bh * a.max_pages + (i < a.max_pages ? i : a.max_pages - 1)];
      sel_pt[SEL_EARLY ? j : 0] = a.page_table[(long long)b * a.max_pages + (e < a.max_pages ? e : a.max_pages - 1)];
    }
  };
  // FUSE: this thread's element of the query, asked for early too (no branch around the load: all threads read)
  uint32_t q_raw = 0u;
  if (FUSE && all_heads) {
    if (SEL_EARLY) ask_selection();
    q_raw = (uint32_t)a.q[(long long)bh * 128 + (tid & 127)];
    __builtin_amdgcn_sched_barrier(0);               // these loads are issued before anything below waits for the lengths
  }
  int P = n > 0 ? (n + TW_PAGE - 1) / TW_PAGE : 0;
  if (P > a.max_pages) P = a.max_pages;
  const int ntok = P * TW_PAGE < n ? P * TW_PAGE : n;
  const int nwords = (ntok + 31) >> 5;
  int count;
  if (FUSE == 2) {
    int P2;
    tw_select_sizes<TW_PAGE>(n, budget_b, a.max_pages, a.max_sel, &P2, &count);
  } else {
    count = a.sel_count[bh];
    if (count > a.max_sel) count = a.max_sel;
    if (count < 0) count = 0;
  }
  const int N = TOK ? count : count * TW_PAGE;
  if (N <= a.n_above || N > a.n_upto) return;     // another launch's head (block-uniform)
  if (FUSE && !all_heads) {
    if (SEL_EARLY) ask_selection();
    q_raw = (uint32_t)a.q[(long long)bh * 128 + (tid & 127)];
  }
  const float* row = a.scores + (long long)bh * a.cand_stride;
  const int c0 = tid * EPT;
  TW_STAMP(0);

  __shared__ unsigned long long histM[HP_NB];
  __shared__ uint32_t histC[HP_NB];
  __shared__ unsigned long long cand_mass[HP_CAP];
  __shared__ uint32_t cand_key[HP_CAP];
  __shared__ uint32_t big_s[HP_BITMAP_WORDS + HP_USTAGE];   // position bitmap, then the union list on its way out
  uint32_t* const bitmap = big_s;                            // (FUSE: first the scores on their way to their owners)
  int32_t* const ustage = (int32_t*)(big_s + HP_BITMAP_WORDS);
  __shared__ unsigned long long tail_s[NW];
  __shared__ uint32_t ws32[16];
  __shared__ float redf[NW];
  __shared__ uint32_t sh_n, sh_kept, sh_T, sh_last;

  __shared__ int32_t pages_s[FUSE == 2 ? 512 : 1];   // FUSE == 2: the head's page list ...
  __shared__ int32_t pool_s[FUSE == 2 ? 512 : 1];    // ... and the pages' places in the pool
  if (FUSE == 2) {
    static_assert(4096 + SEL_NB + 2 * SEL_CAP <= HP_BITMAP_WORDS + HP_USTAGE, "the selection's arrays lie in big_s");
    int32_t* const out = a.sel_pages_w + (long long)bh * a.max_sel;
    const int32_t* const ptab = a.page_table + (long long)b * a.max_pages;
    if (tid == 0) a.sel_count_w[bh] = count;
    if (count == P) {                               // the budget covers the sequence (block-uniform)
      for (int i = tid; i < P; i += NT) { out[i] = i; pages_s[i] = i; pool_s[i] = ptab[i]; }
    } else if (count > 0) {
      if (SEL_EARLY) {
        tw_select_row<NT, 30, SEL_E, true>(nullptr, P, count, a.max_sel, out, pages_s, big_s, big_s + 4096, big_s + 4096 + SEL_NB,
                                           (int32_t*)(big_s + 4096 + SEL_NB + SEL_CAP), sel_pt, pool_s, sel_pre);
      } else {
        // page-table entries of the pages this thread will list, in flight while the threshold is found
        const int E = (P + NT - 1) / NT;
#pragma unroll
        for (int e = 0; e < SEL_E; ++e) { const int i = tid * E + e; sel_pt[FUSE == 2 ? e : 0] = ptab[i < P ? i : P - 1]; }
        tw_select_row<NT, 30, SEL_E, false>(a.bounds + (long long)bh * a.max_pages, P, count, a.max_sel, out, pages_s, big_s,
                                            big_s + 4096, big_s + 4096 + SEL_NB, (int32_t*)(big_s + 4096 + SEL_NB + SEL_CAP),
                                            sel_pt, pool_s);
      }
    }
    __syncthreads();                                // list complete; big_s free for the scores
  }

  // ---- scores into registers; logical pages of the owned slots
  // (loads do not wait for the list length: anything inside the row is readable, slots at or
  //  beyond N are masked afterwards)
  constexpr int NPG = TOK ? EPT : (EPT + 15) / 16; // pages a thread's slots fall into (a part of one if EPT < 16); TOK: one token per slot
  float s[EPT];
  int pg[NPG];
  if (FUSE) {
    static_assert(NT * EPT <= (HP_BITMAP_WORDS + HP_USTAGE), "scores of a row must fit the staging array");
    float* const sc_s = (float*)big_s;
    __shared__ int qi_s[1][32];
    __shared__ float qred[4];
    __shared__ float qc_s[1];
    // this wave's share of the list: lane k holds its k-th page (at most EPT * 4 <= 32 of them)
    constexpr int UF = NT >= 1024 ? 8 : 4;            // pages in flight per wave (register budget)
    const int ppw = ((count + NW - 1) / NW + UF - 1) & ~(UF - 1);
    const int first = __builtin_amdgcn_readfirstlane(wave) * ppw;   // (scalar: the loop below is wave-uniform)
    int my_lp = -1, my_pool = -1;
    if (lane < ppw && first + lane < count) {
      my_lp = FUSE == 2 ? pages_s[first + lane] : a.sel_pages[(long long)bh * a.max_sel + first + lane];
      if (my_lp >= 0 && my_lp < P) {
        const int pp = FUSE == 2 ? pool_s[first + lane] : a.page_table[(long long)b * a.max_pages + my_lp];
        if (pp >= 0 && pp < a.pool_pages) my_pool = pp;
      }
    }
    int npages = count - first;
    npages = npages < 0 ? 0 : (npages > ppw ? ppw : npages);
    tw_quantize_q1(tid < 128 ? __uint_as_float(q_raw << 16) : 0.f, qi_s, qred, qc_s);
    const int j = lane & 3, g = h / G;
    int qw[8], qs = 0;
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      qw[k] = qi_s[0][8 * j + k];
      qs = __builtin_amdgcn_sdot4(qw[k], 0x01010101, qs, false);
    }
    const float qsf = (float)qs, cc = qc_s[0];
#pragma unroll 1
    for (int k0 = 0; k0 < npages; k0 += UF) {
      // UF pages per round: all their loads first (unconditional: lanes past the wave's last page hold pool -1 and
      // read pool page 0), then the arithmetic; every lane of a quad stores the token's score (same word), so the
      // round has no branches and the loads stay together.  Slots past the list's end get -inf (inside the array:
      // NW * ppw <= NT * EPT / 16 pages).
      uint4 nib[UF];
      uint32_t meta[UF];
      int lpk[UF], plk[UF];
#pragma unroll
      for (int kk = 0; kk < UF; ++kk) {
        lpk[kk] = __builtin_amdgcn_readlane(my_lp, (k0 + kk) & 63);
        plk[kk] = __builtin_amdgcn_readlane(my_pool, (k0 + kk) & 63);
        const long long blk = ((long long)(plk[kk] >= 0 ? plk[kk] : 0) * a.Hkv + g) * 64;
        nib[kk] = a.kq_pool[blk + lane];
        meta[kk] = a.kq_meta[blk + lane];
      }
#pragma unroll
      for (int kk = 0; kk < UF; ++kk) {
        int u[8];
        u[0] = nib[kk].x & 0x0F0F0F0F; u[1] = (nib[kk].x >> 4) & 0x0F0F0F0F;
        u[2] = nib[kk].y & 0x0F0F0F0F; u[3] = (nib[kk].y >> 4) & 0x0F0F0F0F;
        u[4] = nib[kk].z & 0x0F0F0F0F; u[5] = (nib[kk].z >> 4) & 0x0F0F0F0F;
        u[6] = nib[kk].w & 0x0F0F0F0F; u[7] = (nib[kk].w >> 4) & 0x0F0F0F0F;
        const bool valid = plk[kk] >= 0 && lpk[kk] * TW_PAGE + (lane >> 2) < n;
        const float T = tw_token_sum(meta[kk], tw_group_dot(qw, u, 0), qsf);
        sc_s[(first + k0 + kk) * TW_PAGE + (lane >> 2)] = valid ? __fmul_rn(T, cc) : -__builtin_inff();
      }
    }
    __syncthreads();
#pragma unroll
    for (int v = 0; v < EPT / 4; ++v) {
      const float4 x = *(const float4*)(sc_s + c0 + 4 * v);
      s[4 * v] = x.x; s[4 * v + 1] = x.y; s[4 * v + 2] = x.z; s[4 * v + 3] = x.w;
    }
    __syncthreads();                               // the bitmap, cleared below, lies in the same words
  } else
#pragma unroll
  for (int v = 0; v < EPT / 4; ++v) {              // clamped, unconditional: all loads go out together
    const int cc = c0 + 4 * v < a.cand_stride ? c0 + 4 * v : a.cand_stride - 4;
    const float4 x = *(const float4*)(row + cc);
    s[4 * v] = x.x; s[4 * v + 1] = x.y; s[4 * v + 2] = x.z; s[4 * v + 3] = x.w;
  }
  if (TOK) {
#pragma unroll
    for (int v = 0; v < EPT / 4; ++v) {
      const int cc = c0 + 4 * v < a.max_sel ? c0 + 4 * v : a.max_sel - 4;
      const int4 x = *(const int4*)(a.sel_pages + (long long)bh * a.max_sel + cc);
      pg[(4 * v) % NPG] = x.x; pg[(4 * v + 1) % NPG] = x.y; pg[(4 * v + 2) % NPG] = x.z; pg[(4 * v + 3) % NPG] = x.w;
    }
  } else {
#pragma unroll
    for (int v = 0; v < NPG; ++v) {
      const int pi = (c0 >> 4) + v < a.max_sel ? (c0 >> 4) + v : a.max_sel - 1;
      pg[v] = FUSE == 2 ? pages_s[pi] : a.sel_pages[(long long)bh * a.max_sel + pi];
    }
  }
#pragma unroll
  for (int e = 0; e < EPT; ++e) s[e] = (c0 + e < N) ? s[e] : -__builtin_inff();
  for (int i = tid; i < HP_NB; i += NT) { histM[i] = 0; histC[i] = 0; }
  for (int i = tid; i < nwords; i += NT) bitmap[i] = 0;
  if (tid == 0) { sh_n = 0; sh_kept = 0; }

  float m = s[0];
#pragma unroll
  for (int e = 1; e < EPT; ++e) m = fmaxf(m, s[e]);
  m = tw_wave_max_f(m);
  if (lane == 0) redf[wave] = m;
  __syncthreads();
  m = redf[0];
#pragma unroll
  for (int w = 1; w < NW; ++w) m = fmaxf(m, redf[w]);
  TW_STAMP(1);

  uint32_t T = 0;
  bool searching;
  if (!(m > -__builtin_inff())) { T = 0xFFFFFFFFu; searching = false; }
  else if (a.p >= 1.0f) { T = kKeyNegInf + 1u; searching = false; }
  else searching = true;

  if (searching) {                                 // block-uniform
    // rank and numerator of every score: computed once and kept, or (512-thread workgroups, which are there
    // to fit more of them on a CU) recomputed from the score where needed - a few instructions that save
    // 2 * EPT registers
    constexpr bool RECOMP = NT <= 512;
    uint32_t rk[RECOMP ? 1 : EPT];
    float ef[RECOMP ? 1 : EPT];
    if (!RECOMP) {
#pragma unroll
      for (int e = 0; e < EPT; ++e) rk[RECOMP ? 0 : e] = hp_rank(m, s[e], &ef[RECOMP ? 0 : e]);
    }
    auto rank_of = [&](int e) -> uint32_t { return RECOMP ? hp_rank_only(m, s[e]) : rk[RECOMP ? 0 : e]; };
    auto numer_of = [&](int e) -> float { return RECOMP ? hp_numer(m, s[e]) : ef[RECOMP ? 0 : e]; };
    uint32_t rlo = 0, pop = 0;
    int shift = 16, pass = 0;
    unsigned long long A = 0, target = 0;
#pragma unroll 1
    for (;;) {
      if (pass > 0) {
        for (int i = tid; i < HP_NB; i += NT) { histM[i] = 0; histC[i] = 0; }
        __syncthreads();
      }
      unsigned long long below = 0;                // mass past the end of the interval (pass 0 only)
#pragma unroll
      for (int e = 0; e < EPT; ++e) {
        const uint32_t r = rank_of(e);
        if (r != HP_NONE && r >= rlo) {
          const uint32_t bk = (r - rlo) >> shift;
          const unsigned long long w = hp_fix(numer_of(e));
          if (bk < HP_NB) { atomicAdd(&histM[bk], w); atomicAdd(&histC[bk], 1u); }
          else below += w;
        }
      }
      if (pass == 0) {
        below = tw_wave_scan_u64(below);
        if (lane == 63) tail_s[wave] = below;
      }
      __syncthreads();
      TW_STAMP(2 + pass);
      // every wave scans the 512 buckets on its own: lane l owns buckets 8l .. 8l+7
      unsigned long long mb[8], mine = 0;
#pragma unroll
      for (int k = 0; k < 8; ++k) { mb[k] = histM[8 * lane + k]; mine += mb[k]; }
      const unsigned long long incl = tw_wave_scan_u64(mine);
      const unsigned long long total = __shfl(incl, 63, 64);
      if (pass == 0) {
        unsigned long long Z = total;
#pragma unroll
        for (int w = 0; w < NW; ++w) Z += tail_s[w];
        const double t = ceil((double)a.p * (double)Z);
        target = t < 1.0 ? 1ull : (unsigned long long)t;
        if (target > Z) target = Z;
      }
      const unsigned long long before = A + incl - mine;
      const bool hit = before < target && before + mine >= target;
      const unsigned long long bal = __ballot(hit);
      bool more = false;
      if (bal == 0 && pass == 0) {
        // not enough mass in the fine range: go on with everything below it
        A += total;
        rlo = HP_FINE_END; shift = 18;
        more = true;
      } else if (bal == 0) {
        pop = 0xFFFFFFFFu;                          // unreachable: the interval holds the crossing by construction
      } else {
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
        rlo += (uint32_t)bucket << shift;
        if (pop > HP_CAP && shift > 0) { shift = shift >= 9 ? shift - 9 : 0; more = true; }
      }
      ++pass;
      if (!more) break;                             // same decision in every wave
      __syncthreads();                              // all scans done before the histogram is cleared
    }
    // the threshold lies among the `pop` scores with rank in [rlo, rlo + (1 << shift))
    const uint32_t rhi = rlo + (1u << shift) - 1u;
    const bool small = pop <= HP_CAP;
    uint32_t kmin = 0xFFFFFFFFu;
#pragma unroll
    for (int e = 0; e < EPT; ++e) {
      const uint32_t r = rank_of(e);
      if (r != HP_NONE && r >= rlo && r <= rhi) {
        const uint32_t k = tw_float_key(s[e]);
        kmin = k < kmin ? k : kmin;
        if (small) {
          const uint32_t at = atomicAdd(&sh_n, 1u);
          if (at < HP_CAP) { cand_key[at] = k; cand_mass[at] = hp_fix(numer_of(e)); }
        }
      }
    }
    if (!small) {                                   // > HP_CAP scores within one rank: keep them all
      kmin = ~tw_wave_max_u32(~kmin);
      if (lane == 0) redf[wave] = __uint_as_float(kmin);
    }
    __syncthreads();
    TW_STAMP(8);
    if (wave == 0) {                                // one wave resolves; the others wait at the barrier
      if (small) {
        // lane x takes candidate x: mass of all candidates at least as large as it
        const uint32_t cn = sh_n < HP_CAP ? sh_n : HP_CAP;
        const uint32_t kx = lane < (int)cn ? cand_key[lane] : 0u;
        unsigned long long S = 0;
#pragma unroll 4
        for (uint32_t j = 0; j < cn; ++j) {
          const uint32_t kj = cand_key[j];
          const unsigned long long wj = cand_mass[j];
          S += kj >= kx ? wj : 0ull;
        }
        const uint32_t best = (lane < (int)cn && A + S >= target) ? kx : 0u;
        T = tw_wave_max_u32(best);
      } else {
        uint32_t r = __float_as_uint(redf[0]);
#pragma unroll
        for (int w = 1; w < NW; ++w) { const uint32_t y = __float_as_uint(redf[w]); r = y < r ? y : r; }
        T = r;
      }
      if (lane == 0) sh_T = T;
    }
    __syncthreads();
    T = sh_T;
    TW_STAMP(9);
  }

  // ---- kept flags, count, optional ascending list; bitmap over token positions
  uint32_t cnt = 0, keep = 0;
#pragma unroll
  for (int e = 0; e < EPT; ++e) {
    const bool k = (c0 + e < N) && tw_float_key(s[e]) >= T;
    keep |= (k ? 1u : 0u) << e;
    cnt += k ? 1u : 0u;
  }
  uint32_t pos = 0;
  if (a.kept_idx) {                                // ordered positions need a scan over the block
    uint32_t total;
    const uint32_t incl = tw_block_scan_u32(cnt, ws32, &total);
    pos = incl - cnt;
    if (tid == 0) sh_kept = total;
  } else {
    const uint32_t wsumc = tw_wave_scan_u32(cnt);
    if (lane == 63 && wsumc) atomicAdd(&sh_kept, wsumc);
  }
  if (TOK) {
    int32_t* out = a.kept_idx ? a.kept_idx + (long long)bh * a.kept_stride : nullptr;
#pragma unroll
    for (int e = 0; e < EPT; ++e) {
      if ((keep >> e) & 1u) {                       // kept => valid score => a token inside the sequence
        const int tok = pg[e % NPG];
        if (tok < HP_BITMAP_WORDS * 32) atomicOr(&bitmap[tok >> 5], 1u << (tok & 31));
        if (out) { if (pos < (uint32_t)a.kept_stride) out[pos] = tok; ++pos; }
      }
    }
  } else
#pragma unroll
  for (int v = 0; v < NPG; ++v) {
    constexpr int PB = EPT < 16 ? EPT : 16;        // slots of this thread inside page v
    const uint32_t mask = (keep >> (16 * v)) & ((1u << PB) - 1u);
    if (mask) {
      const int tok0 = pg[v] * TW_PAGE + (EPT < 16 ? (c0 & 15) : 0);
      if (tok0 + 15 < HP_BITMAP_WORDS * 32) atomicOr(&bitmap[tok0 >> 5], mask << (tok0 & 31));
      if (a.kept_idx) {
        int32_t* out = a.kept_idx + (long long)bh * a.kept_stride;
#pragma unroll
        for (int e = 0; e < PB; ++e)
          if ((mask >> e) & 1u) { if (pos < (uint32_t)a.kept_stride) out[pos] = tok0 + e; ++pos; }
      }
    }
  }
  __syncthreads();
  uint32_t* bm = a.bitmaps + (long long)bh * a.words_stride;
#ifdef TW_FORMAL_ORDER
  // Measurement build: the hand-off written with the memory model's own pair - plain stores, a workgroup
  // barrier, one agent-scope acq_rel read-modify-write by thread 0 (release: everything the block wrote is
  // made visible to the agent first; acquire: nothing the reader loads afterwards may be stale).
  for (int i = tid; i < nwords; i += NT) bm[i] = bitmap[i];
  if (tid == 0) {
    uint32_t kc = sh_kept;
    if (a.kept_idx && kc > (uint32_t)a.kept_stride) { atomicOr(a.status, TW_STATUS_KEPT_TRUNCATED); kc = a.kept_stride; }
    a.kept_count[bh] = (int32_t)kc;
  }
  const int gi = b * a.Hkv + h / G;
  __syncthreads();
  if (tid == 0)
    sh_last = __hip_atomic_fetch_add(a.arrive + gi * TW_CTR, 1u, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_AGENT) == (uint32_t)(G - 1) ? 1u : 0u;
  __syncthreads();
#else
  // device-scope (write-through) stores: the group's last head reads these words from another CU
  for (int i = tid; i < nwords; i += NT) __hip_atomic_store(bm + i, bitmap[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  if (tid == 0) {
    uint32_t kc = sh_kept;
    if (a.kept_idx && kc > (uint32_t)a.kept_stride) { atomicOr(a.status, TW_STATUS_KEPT_TRUNCATED); kc = a.kept_stride; }
    a.kept_count[bh] = (int32_t)kc;
  }
  TW_STAMP(12);

  // ---- the last head of the KV head's group to get here turns the G bitmaps into the sorted union
  const int gi = b * a.Hkv + h / G;
  // Ordering without cache-wide fences: the bitmap words are stored and loaded with agent-scope atomics
  // (write-through stores, loads that bypass the caches that are not shared by all compute units), every
  // thread waits for the acknowledgement of its own stores (a workgroup barrier alone does not), the barrier
  // then collects the block, and only after it does thread 0 count the arrival.  The last head of the group
  // therefore finds every earlier head's words in place.  (The memory model's own form of this hand-off - plain
  // stores and an acq_rel counter, -DTW_FORMAL_ORDER - writes back and invalidates the whole L2 at every arrival.)
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
  if (tid == 0)
    sh_last = __hip_atomic_fetch_add(a.arrive + gi * TW_CTR, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == (uint32_t)(G - 1) ? 1u : 0u;
  __syncthreads();
#endif
  if (!sh_last) return;
  TW_STAMP_IF(gi == 0, 14);
  if (tid == 0) __hip_atomic_store(a.arrive + gi * TW_CTR, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // ready for the next call
  // OR of the group's bitmaps into LDS (this block's own bitmap is no longer needed there): coalesced,
  // four words per thread and bitmap in flight
  const uint32_t* bmg = a.bitmaps + ((long long)(b * a.Hq + (h / G) * G)) * a.words_stride;
  for (int base = 0; base < nwords; base += 4 * NT) {
    uint32_t x[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      x[k] = 0;
      if (base + k * NT < nwords) {                  // block-uniform
        const int i = base + k * NT + tid;
        const int wi = i < nwords ? i : 0;
#pragma unroll
        for (int hh = 0; hh < G; ++hh)
#ifdef TW_FORMAL_ORDER
          x[k] |= bmg[(long long)hh * a.words_stride + wi];
#else
          x[k] |= __hip_atomic_load(bmg + (long long)hh * a.words_stride + wi, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#endif
      }
    }
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const int i = base + k * NT + tid;
      if (i < nwords) bitmap[i] = x[k];
    }
  }
  __syncthreads();
  TW_STAMP_IF(gi == 0, 15);
  int32_t* uout = a.union_idx + (long long)gi * a.union_stride;
  uint32_t utotal;
  // (block-uniform choice: long sequences - more than two bitmap words per thread - take the wave-cooperative
  //  listing; with fewer words per thread the plain per-thread walk is as quick and needs fewer registers, which
  //  is what the 512-thread workgroups are short of)
  if (NT >= 1024 && nwords > 2 * NT) {
    // Wave w owns the contiguous words [w * wpw, (w + 1) * wpw) and takes them 64 at a time, one word per lane.  The
    // set bits of a round are listed either by every lane walking its own word (scattered kept tokens: few bits per
    // word) or, when fewer words are non-empty than the fullest word has bits (clustered heavy hitters: a few words
    // of 32), word by word with one lane per bit - two words at a time, one per half wave.
    const int wpw = (((nwords + NW - 1) / NW) + 63) & ~63;
    const int wbase = wave * wpw;
    uint32_t ucnt = 0;
    for (int r = 0; r < wpw; r += 64) {
      const int i = wbase + r + lane;
      ucnt += i < nwords ? __popc(bitmap[i]) : 0;
    }
    ucnt = tw_wave_scan_u32(ucnt);
    if (lane == 63) ws32[wave] = ucnt;
    __syncthreads();
    uint32_t run = 0;
    utotal = 0;
  #pragma unroll
    for (int w = 0; w < NW; ++w) { const uint32_t t = ws32[w]; run += w < wave ? t : 0u; utotal += t; }
    TW_STAMP_IF(gi == 0, 16);
    // positions staged in LDS and copied out coalesced when they fit (the usual case; block-uniform), else stored directly
    const bool staged = utotal <= (uint32_t)HP_USTAGE;
    auto put = [&](uint32_t pos, int tok) {
      if (staged) ustage[pos] = tok;
      else if (pos < (uint32_t)a.union_stride) uout[pos] = tok;
    };
    for (int r = 0; r < wpw; r += 64) {               // wave-uniform trip count
      const int i = wbase + r + lane;
      uint32_t x = i < nwords ? bitmap[i] : 0u;
      const uint32_t c = __popc(x);
      const uint32_t incl = tw_wave_scan_u32(c);
      const uint32_t upos0 = run + incl - c;
      run += __shfl(incl, 63, 64);
      unsigned long long nz = __ballot(x != 0);
      if (nz == 0) continue;                           // wave-uniform
      const uint32_t maxc = tw_wave_max_u32(c);
      if ((uint32_t)__popcll(nz) * 2 >= maxc) {        // every lane its own word
        uint32_t upos = upos0;
        while (x) {
          const int bit = __ffs(x) - 1;
          x &= x - 1;
          put(upos++, i * 32 + bit);
        }
      } else {                                         // two non-empty words per step, one lane per bit
        const int half = lane >> 5, bit = lane & 31;
        while (nz) {                                   // wave-uniform
          const int s0 = __ffsll((long long)nz) - 1;
          nz &= nz - 1;
          int s1 = -1;
          if (nz) { s1 = __ffsll((long long)nz) - 1; nz &= nz - 1; }
          const int src = half ? s1 : s0;
          const uint32_t xw = (uint32_t)__shfl((int)x, src < 0 ? 0 : src, 64);
          const uint32_t ow = (uint32_t)__shfl((int)upos0, src < 0 ? 0 : src, 64);
          if (src >= 0 && ((xw >> bit) & 1u))
            put(ow + __popc(xw & ((1u << bit) - 1u)), (wbase + r + src) * 32 + bit);
        }
      }
    }
    if (staged) {
      __syncthreads();
      const uint32_t lim = utotal < (uint32_t)a.union_stride ? utotal : (uint32_t)a.union_stride;
      for (uint32_t i = tid; i < lim; i += NT) uout[i] = ustage[i];
    }
  } else {
    // thread t owns the contiguous words [t * wpt, (t + 1) * wpt): ascending output positions
    const int wpt = (nwords + NT - 1) / NT;
    const int w0 = tid * wpt, w1 = w0 + wpt < nwords ? w0 + wpt : nwords;
    uint32_t ucnt = 0;
    for (int i = w0; i < w1; ++i) ucnt += __popc(bitmap[i]);
    const uint32_t uincl = tw_block_scan_u32(ucnt, ws32, &utotal);
    TW_STAMP_IF(gi == 0, 16);
    uint32_t upos = uincl - ucnt;
    if (utotal <= (uint32_t)HP_USTAGE) {               // block-uniform; the usual case
      // positions staged in LDS, then copied out coalesced: a dense word costs its thread 32 scattered
      // stores otherwise, one store instruction of the whole wave each (1.5 us of the kernel's tail)
      for (int i = w0; i < w1; ++i) {
        uint32_t x = bitmap[i];
        while (x) {
          const int bit = __ffs(x) - 1;
          x &= x - 1;
          ustage[upos++] = i * 32 + bit;
        }
      }
      __syncthreads();
      const uint32_t lim = utotal < (uint32_t)a.union_stride ? utotal : (uint32_t)a.union_stride;
      for (uint32_t i = tid; i < lim; i += NT) uout[i] = ustage[i];
    } else {
      for (int i = w0; i < w1; ++i) {
        uint32_t x = bitmap[i];
        while (x) {
          const int bit = __ffs(x) - 1;
          x &= x - 1;
          if (upos < (uint32_t)a.union_stride) uout[upos] = i * 32 + bit;
          ++upos;
        }
      }
    }
  }
  if (tid == 0) {
    if (utotal > (uint32_t)a.union_stride) { atomicOr(a.status, TW_STATUS_UNION_TRUNCATED); utotal = a.union_stride; }
    a.union_count[gi] = (int32_t)utotal;
  }
  TW_STAMP_IF(gi == 0, 13);
}

// ------------------------------------------------------------------ launches
int pages_per_wave(long long total_pages_all_rows, int count_bound) {
  // 4..64 pages per wave, at least ~8192 waves chip-wide (one per wave slot: measured at
  // 65536 candidate pages, 8 pages per wave beat 16 by 15 %; ragged batches whose bound is far
  // above the mean list length do best with long waves, fewer of which are empty)
  int pw = 64;
  while (pw > 4 && total_pages_all_rows / pw < 8192) pw >>= 1;
  while (pw > 4 && pw / 2 >= count_bound) pw >>= 1;
  return pw;
}

template <int NH, bool FULL>
void launch_score(const ScoreArgs& a, dim3 grid, bool dots, int bits, hipStream_t s) {
  // pages in flight per wave: 4, fewer when 8 heads share a page (register budget)
  if (bits == 2) {
    if (dots) TW_LAUNCH((int4_score_kernel<NH, FULL, true, 2, 2>), grid, dim3(256), 0, s, a);
    else      TW_LAUNCH((int4_score_kernel<NH, FULL, false, 2, 2>), grid, dim3(256), 0, s, a);
  } else if (bits == 8) {
    if (dots) TW_LAUNCH((int4_score_kernel<NH, FULL, true, 2, 8>), grid, dim3(256), 0, s, a);
    else      TW_LAUNCH((int4_score_kernel<NH, FULL, false, 2, 8>), grid, dim3(256), 0, s, a);
  }
  else if (dots) TW_LAUNCH((int4_score_kernel<NH, FULL, true, 2>), grid, dim3(256), 0, s, a);
  else if (NH < 8) TW_LAUNCH((int4_score_kernel<NH, FULL, false, 4>), grid, dim3(256), 0, s, a);
  else TW_LAUNCH((int4_score_kernel<NH, FULL, false, 2>), grid, dim3(256), 0, s, a);
}

int run_score(const twilight_kv_t* kv, const TwDims& d, const void* q, const int32_t* sel_pages,
              const int32_t* sel_count, int32_t max_sel, float* scores, int32_t* dots, uint32_t* arrive,
              uint32_t* headmax, hipStream_t s, const uint32_t* chmask = nullptr) {
  ScoreArgs a;
  a.arrive = arrive; a.headmax = headmax; a.chmask = chmask;
  a.q = (const uint16_t*)q; a.sel_pages = sel_pages; a.sel_count = sel_count;
  a.page_table = kv->page_table; a.seq_lens = kv->seq_lens;
  a.kq_pool = (const uint4*)kv->kq_pool; a.kq_meta = (const uint32_t*)kv->kq_meta;
  a.scores = scores; a.dots = dots;
  a.Hq = d.Hq; a.Hkv = d.Hkv; a.max_pages = d.max_pages; a.max_sel = max_sel;
  a.pool_pages = d.pool_pages;
  const bool full = sel_pages == nullptr;
  const int bound = full ? d.max_pages : max_sel;
  a.cand_stride = bound * TW_PAGE;
  a.pw = pages_per_wave((long long)bound * d.batch * (full ? d.Hkv : d.Hq), bound);
#ifdef TW_TUNING                                 // tuning builds only: the shipped library reads no environment
  static const int pw_env = getenv("TW_INT4_PW") ? atoi(getenv("TW_INT4_PW")) : 0;
  static const int x_env = getenv("TW_INT4_X") ? atoi(getenv("TW_INT4_X")) : 0;
  static const bool valu_only = getenv("TW_INT4_VALU") != nullptr;   // vector-ALU kernel for every G
#else
  constexpr int pw_env = 0, x_env = 0;
  constexpr bool valu_only = false;
#endif
  if (pw_env >= 4 && pw_env <= 64) a.pw = pw_env;
  dim3 grid((bound + 4 * a.pw - 1) / (4 * a.pw), d.batch * (full ? d.Hkv : d.Hq));
  a.rotate = 0;
  if (!full) {
    // Per-head page lists: at most 8 pages per wave; rows of more than 8 chunks get a grid a multiple of 8 wide
    // (one column per XCD, see the kernel) and at most about 16384 workgroups - batches of many heads have
    // lists far shorter than the row bound, and their workgroups loop over the chunks beyond the grid
    if (!(pw_env >= 4 && pw_env <= 64) && a.pw > 8) a.pw = 8;
    int x = (bound + 4 * a.pw - 1) / (4 * a.pw);
    if (x > 8) {
      long long cap = 16384 / ((long long)d.batch * d.Hq);
      if (cap > x) cap = x;
      x = cap < 8 ? 8 : (int)(cap & ~7ll);
    }
    if (x_env > 0) x = x_env;
    grid.x = x;
    a.rotate = (x & 7) == 0 ? 1 : 0;
  }
  tw_prof_before(TW_K_INT4_SCORE, s);
  if (!full) launch_score<1, false>(a, grid, dots != nullptr, d.bits, s);
  else if (d.G >= 4 && d.bits == 4 && !valu_only) {               // matrix-core kernel: 4 or 8 heads share every page
    // 8 pages in flight per wave (the kernel needs few registers, so 4 to 7 waves per SIMD stay resident)
    if (d.G == 4) {
      if (dots) TW_LAUNCH((int4_score_mfma_kernel<1, true, 4>), grid, dim3(256), 0, s, a);
      else      TW_LAUNCH((int4_score_mfma_kernel<1, false, 8>), grid, dim3(256), 0, s, a);
    } else {
      if (dots) TW_LAUNCH((int4_score_mfma_kernel<2, true, 4>), grid, dim3(256), 0, s, a);
      else      TW_LAUNCH((int4_score_mfma_kernel<2, false, 8>), grid, dim3(256), 0, s, a);
    }
  } else switch (d.G) {
    case 1: launch_score<1, true>(a, grid, dots != nullptr, d.bits, s); break;
    case 2: launch_score<2, true>(a, grid, dots != nullptr, d.bits, s); break;
    case 4: launch_score<4, true>(a, grid, dots != nullptr, d.bits, s); break;
    default: launch_score<8, true>(a, grid, dots != nullptr, d.bits, s); break;
  }
  return tw_prof_after(s);
}


template <int NT, int EPT, bool TOK, int FUSE>
void launch_topp_one(const HeadArgs& f, int G, dim3 grid, hipStream_t s) {
  switch (G) {
    case 1: TW_LAUNCH((topp_head_kernel<NT, EPT, 1, TOK, FUSE>), grid, dim3(NT), 0, s, f); break;
    case 2: TW_LAUNCH((topp_head_kernel<NT, EPT, 2, TOK, FUSE>), grid, dim3(NT), 0, s, f); break;
    case 4: TW_LAUNCH((topp_head_kernel<NT, EPT, 4, TOK, FUSE>), grid, dim3(NT), 0, s, f); break;
    default: TW_LAUNCH((topp_head_kernel<NT, EPT, 8, TOK, FUSE>), grid, dim3(NT), 0, s, f); break;
  }
}

// Register-resident top-p over rows of at most 8192 candidates (cand_stride = row bound).
//  - few heads: one 1024-thread workgroup per head (4 or 8 candidates per thread);
//  - more heads than CUs and rows of at most 4096 candidates: 512-thread workgroups, two to a CU (a 1024-thread
//    workgroup has a CU to itself at this register count: 8 x 32 x 4 = 1024 heads took 35.8 us that way, 22.9 us so);
//  - many heads with a bound above 4096 candidates (ragged batches): heads of at most 4096 candidates go to a
//    512-thread launch of their own, the longer ones to the 1024-thread launch.
// FUSE: the kernels score the candidates themselves (page lists, 4-bit codes).
template <bool TOK, int FUSE = 0>
int launch_topp(HeadArgs f, const TwDims& d, int cand_stride, hipStream_t s) {
  const dim3 grid(d.Hq, d.batch);
  const long long heads = (long long)d.batch * d.Hq;
  f.remap = (FUSE != 0 && ((long long)d.batch * d.Hkv) % 8 == 0) ? 1 : 0;
  f.n_above = -1; f.n_upto = cand_stride;
  if (cand_stride > 4096 && heads > 2ll * tw_num_cus()) {
    f.n_upto = 4096;
    tw_prof_before(FUSE == 2 ? TW_K_SELECT_SCORE_TOPP : (FUSE == 1 ? TW_K_SCORE_TOPP : TW_K_TOPP), s);
    launch_topp_one<512, 8, TOK, FUSE>(f, d.G, grid, s);
    if (int e = tw_prof_after(s)) return e;
    f.n_above = 4096; f.n_upto = cand_stride;
  }
  tw_prof_before(FUSE == 2 ? TW_K_SELECT_SCORE_TOPP : (FUSE == 1 ? TW_K_SCORE_TOPP : TW_K_TOPP), s);
  if (cand_stride <= 4096 && heads > tw_num_cus()) launch_topp_one<512, 8, TOK, FUSE>(f, d.G, grid, s);
  else if (cand_stride <= 4096) launch_topp_one<1024, 4, TOK, FUSE>(f, d.G, grid, s);
  else launch_topp_one<1024, 8, TOK, FUSE>(f, d.G, grid, s);
  return tw_prof_after(s);
}

}  // namespace


// Channel-sparse estimate of every token of every sequence (the scoring half of the channel-sparse token selector):
// scores [b][Hq][max_pages * 16], tokens at or beyond the sequence's end -inf.
int tw_score_all_tokens_masked(const twilight_kv_t* kv, const TwDims& d, const void* q, const uint32_t* chmask, float* scores,
                               hipStream_t s) {
  return run_score(kv, d, q, nullptr, nullptr, 0, scores, nullptr, nullptr, nullptr, s, chmask);
}

int tw_prune_wide_init(const TwDims& d, const PruneWs& L, void* ws, hipStream_t s);
int tw_prune_wide(const TwDims& d, const PruneWs& L, void* ws, const twilight_kv_t* kv, const int32_t* sel_pages,
                  const int32_t* sel_count, int max_sel, int cand_stride, float p, int32_t* kept_count,
                  int32_t* kept_idx, int kept_stride, int32_t* union_count, int32_t* union_idx, int union_stride,
                  uint32_t* status, hipStream_t s);

// Register-resident per-head kernel: per-head lists of at most 8192 candidates on sequences whose
// position bitmap fits in LDS; everything else takes the multi-workgroup path.
bool tw_prune_uses_head_kernel(const TwDims& d, bool full, int bound_pages) {
  return !full && bound_pages * TW_PAGE <= 1024 * 8 && (long long)d.max_pages * TW_PAGE <= HP_BITMAP_WORDS * 32ll;
}

PruneWs tw_prune_layout(const TwDims& d, int bound_pages, bool full) {
  auto al = [](size_t x) { return (x + 255) & ~(size_t)255; };
  const size_t bh = (size_t)d.batch * d.Hq;
  PruneWs L;
  L.words_stride = (d.max_pages + 1) / 2;
  size_t o = 0;
  L.scores = o;  o += al(bh * (size_t)bound_pages * TW_PAGE * 4);
  const bool head = tw_prune_uses_head_kernel(d, full, bound_pages);
  L.headmax = o; o += head ? 256 : al(bh * HM_SLOTS * TW_CTR * 4);   // (the long-row path clears from here ...)
  L.arrive = o;  o += al((size_t)d.batch * d.Hkv * TW_CTR * 4);
  L.bitmaps = o; o += al(bh * (size_t)L.words_stride * 4);
  if (head) {                                                // the long-row buffers are not needed
    L.ghistM = L.ghistC = L.ucount = L.kdef = L.state = L.ulist = L.segcnt = o;
    L.total = o;
    return L;
  }
  L.ghistM = o;  o += al(bh * 2048 * 8);
  L.ghistC = o;  o += al(bh * 2048 * 4);
  L.ucount = o;  o += al(bh * TW_CTR * 4);
  L.kdef = o;    o += al(bh * TW_CTR * 4);
  L.state = o;   o += al(bh * 48);                       // (... up to here)
  L.ulist = o;   o += al(bh * 4096 * 8);
  L.segcnt = o;  o += al(bh * (size_t)((L.words_stride + 255) / 256) * 4);   // set bits per 256-word segment of a row's bitmap(s)
  L.total = o;
  return L;
}

#ifdef TW_PHASE_TIMING
extern "C" int twilight_debug_stamps_prune(unsigned long long* host_out) {
  return hipMemcpyFromSymbol(host_out, HIP_SYMBOL(tw_dbg_stamps), sizeof(unsigned long long) * 64) == hipSuccess ? 0 : -1;
}
#endif

extern "C" int twilight_int4_score(const twilight_kv_t* kv, const void* q, const int32_t* sel_pages,
                                   const int32_t* sel_count, int32_t max_sel, float* scores, int32_t* dots,
                                   void* stream) {
  TwDims d;
  if (int e = tw_check_kv(kv, &d)) return e;
  if (!q || !scores || !kv->kq_pool || !kv->kq_meta) return TW_EINVAL;
  if (sel_pages && (!sel_count || max_sel <= 0)) return TW_EINVAL;
  return run_score(kv, d, q, sel_pages, sel_count, max_sel, scores, dots, nullptr, nullptr, (hipStream_t)stream);
}

extern "C" int twilight_topp_prune(const twilight_kv_t* kv, const void* q, const int32_t* sel_pages,
                                   const int32_t* sel_count, int32_t max_sel, float p,
                                   int32_t* kept_count, int32_t* kept_idx, int32_t kept_stride,
                                   int32_t* union_count, int32_t* union_idx, int32_t union_stride,
                                   uint32_t* status, void* ws, size_t ws_bytes, void* stream) {
  TwDims d;
  if (int e = tw_check_kv(kv, &d)) return e;
  if (!q || !kept_count || !union_count || !union_idx || !status || !kv->kq_pool || !kv->kq_meta) return TW_EINVAL;
  if (sel_pages && (!sel_count || max_sel <= 0)) return TW_EINVAL;
  if (!(p > 0.f) || p > 1.f || union_stride <= 0 || (kept_idx && kept_stride <= 0)) return TW_EINVAL;
  const bool full = sel_pages == nullptr;
  const int bound = full ? d.max_pages : max_sel;
  if ((long long)bound * TW_PAGE > (1ll << 22)) return TW_EINVAL;   // fixed-point mass headroom
  if (!ws || ws_bytes < tw_prune_layout(d, bound, full).total) return TW_EWORKSPACE;
  hipStream_t s = (hipStream_t)stream;
  const int cand_stride = bound * TW_PAGE;
  const PruneWs L = tw_prune_layout(d, bound, full);
  float* scores = (float*)((char*)ws + L.scores);
  uint32_t* headmax = (uint32_t*)((char*)ws + L.headmax);
  uint32_t* arrive = (uint32_t*)((char*)ws + L.arrive);
  const bool use_head = tw_prune_uses_head_kernel(d, full, bound);

  if (!use_head)
    if (int e = tw_prune_wide_init(d, L, ws, s)) return e;     // clears headmax before the scoring kernel folds into it
  if (int e = run_score(kv, d, q, sel_pages, sel_count, max_sel, scores, nullptr, use_head ? arrive : nullptr,
                        use_head ? nullptr : headmax, s)) return e;
  if (!use_head)
    return tw_prune_wide(d, L, ws, kv, sel_pages, sel_count, max_sel, cand_stride, p, kept_count, kept_idx, kept_stride,
                         union_count, union_idx, union_stride, status, s);

  // per-head page lists short enough for registers and sequences that fit the LDS bitmap: one
  // launch does top-p per head and, in the last head of each group to finish, the group's union
  {
    const int words_stride = L.words_stride;
    uint32_t* bitmaps = (uint32_t*)((char*)ws + L.bitmaps);
    HeadArgs f;
    f.scores = scores; f.sel_pages = sel_pages; f.sel_count = sel_count; f.seq_lens = kv->seq_lens;
    f.kept_count = kept_count; f.kept_idx = kept_idx; f.bitmaps = bitmaps; f.arrive = arrive;
    f.union_count = union_count; f.union_idx = union_idx; f.status = status;
    f.Hq = d.Hq; f.Hkv = d.Hkv; f.max_pages = d.max_pages; f.max_sel = max_sel; f.cand_stride = cand_stride;
    f.kept_stride = kept_stride; f.words_stride = words_stride; f.union_stride = union_stride; f.p = p;
    f.q = nullptr; f.page_table = nullptr; f.kq_pool = nullptr; f.kq_meta = nullptr; f.pool_pages = 0;
    f.bounds = nullptr; f.budget = nullptr; f.sel_pages_w = nullptr; f.sel_count_w = nullptr;
    return launch_topp<false>(f, d, cand_stride, s);
  }
}

// Pruner over per-head page lists with the scoring done inside the top-p kernel (one launch).  The arrival
// counters at `ws` + layout.arrive must be zero: a kernel earlier on the stream clears them.
// bounds != nullptr: the kernel also selects the head's pages from the bounds of all pages ([b][Hq][max_pages],
// with the budgets) and writes the lists to sel_pages / sel_count; else it reads the lists from there.
bool tw_prune_fused_ok(const TwDims& d, int max_sel, bool with_select) {
  if (d.bits != 4 || max_sel <= 0 || !tw_prune_uses_head_kernel(d, false, max_sel)) return false;
  return !with_select || d.max_pages <= 4096;      // the selection's keys share the kernel's LDS staging array
}
int tw_prune_fused(const twilight_kv_t* kv, const TwDims& d, const void* q, const float* bounds, const int32_t* budget,
                   int32_t* sel_pages, int32_t* sel_count, int32_t max_sel, float p, int32_t* kept_count, int32_t* kept_idx,
                   int32_t kept_stride, int32_t* union_count, int32_t* union_idx, int32_t union_stride,
                   uint32_t* status, void* ws, hipStream_t s) {
  const PruneWs L = tw_prune_layout(d, max_sel, false);
  HeadArgs f;
  f.scores = nullptr; f.sel_pages = sel_pages; f.sel_count = sel_count; f.seq_lens = kv->seq_lens;
  f.kept_count = kept_count; f.kept_idx = kept_idx; f.bitmaps = (uint32_t*)((char*)ws + L.bitmaps);
  f.arrive = (uint32_t*)((char*)ws + L.arrive);
  f.union_count = union_count; f.union_idx = union_idx; f.status = status;
  f.Hq = d.Hq; f.Hkv = d.Hkv; f.max_pages = d.max_pages; f.max_sel = max_sel; f.cand_stride = max_sel * TW_PAGE;
  f.kept_stride = kept_stride; f.words_stride = L.words_stride; f.union_stride = union_stride; f.p = p;
  f.q = (const uint16_t*)q; f.page_table = kv->page_table; f.kq_pool = (const uint4*)kv->kq_pool;
  f.kq_meta = (const uint32_t*)kv->kq_meta; f.pool_pages = d.pool_pages;
  f.bounds = bounds; f.budget = budget; f.sel_pages_w = sel_pages; f.sel_count_w = sel_count;
  if (bounds) return launch_topp<false, 2>(f, d, max_sel * TW_PAGE, s);
  return launch_topp<false, 1>(f, d, max_sel * TW_PAGE, s);
}

// ------------------------------------------------------------------ token-list candidates
static int tw_check_tokens(const TwDims& d, int32_t max_cand) {
  if (max_cand <= 0 || (max_cand & 15) || max_cand > 1024 * 8) return TW_EINVAL;
  if ((long long)d.max_pages * TW_PAGE > HP_BITMAP_WORDS * 32ll) return TW_EINVAL;
  return TW_OK;
}

PruneWs tw_prune_layout_tokens(const TwDims& d, int max_cand) {
  auto al = [](size_t x) { return (x + 255) & ~(size_t)255; };
  const size_t bh = (size_t)d.batch * d.Hq;
  PruneWs L;
  L.words_stride = (d.max_pages + 1) / 2;
  size_t o = 0;
  L.scores = o;  o += al(bh * (size_t)max_cand * 4);
  L.headmax = o;
  L.arrive = o;  o += al((size_t)d.batch * d.Hkv * TW_CTR * 4);
  L.bitmaps = o; o += al(bh * (size_t)L.words_stride * 4);
  L.ghistM = L.ghistC = L.ucount = L.kdef = L.state = L.ulist = L.segcnt = o;
  L.total = o;
  return L;
}

static int run_score_tokens(const twilight_kv_t* kv, const TwDims& d, const void* q, const int32_t* cand_tokens,
                            const int32_t* cand_count, int32_t max_cand, float* scores, int32_t* dots,
                            uint32_t* arrive, hipStream_t s) {
  ScoreArgs a;
  a.arrive = arrive; a.headmax = nullptr; a.chmask = nullptr;
  a.q = (const uint16_t*)q; a.sel_pages = cand_tokens; a.sel_count = cand_count;
  a.page_table = kv->page_table; a.seq_lens = kv->seq_lens;
  a.kq_pool = (const uint4*)kv->kq_pool; a.kq_meta = (const uint32_t*)kv->kq_meta;
  a.scores = scores; a.dots = dots;
  a.Hq = d.Hq; a.Hkv = d.Hkv; a.max_pages = d.max_pages; a.max_sel = max_cand; a.cand_stride = max_cand; a.pw = 0; a.rotate = 0;
  a.pool_pages = d.pool_pages;
  // grid as for page lists: rows of more than 8 chunks get a width that is a multiple of 8, cut so that the
  // launch stays near 16384 workgroups; the workgroups loop over the chunks beyond it
  int x = (max_cand + 255) / 256;
  if (x > 8) {
    long long cap = 16384 / ((long long)d.batch * d.Hq);
    if (cap > x) cap = x;
    x = cap < 8 ? 8 : (int)(cap & ~7ll);
  }
  a.rotate = (x & 7) == 0 ? 1 : 0;
  const dim3 grid(x, d.batch * d.Hq);
  tw_prof_before(TW_K_INT4_SCORE, s);
  if (d.bits == 2) {
    if (dots) TW_LAUNCH((int4_score_tokens_kernel<true, 2>), grid, dim3(256), 0, s, a);
    else      TW_LAUNCH((int4_score_tokens_kernel<false, 2>), grid, dim3(256), 0, s, a);
  } else if (d.bits == 8) {
    if (dots) TW_LAUNCH((int4_score_tokens_kernel<true, 8>), grid, dim3(256), 0, s, a);
    else      TW_LAUNCH((int4_score_tokens_kernel<false, 8>), grid, dim3(256), 0, s, a);
  } else {
    if (dots) TW_LAUNCH((int4_score_tokens_kernel<true, 4>), grid, dim3(256), 0, s, a);
    else      TW_LAUNCH((int4_score_tokens_kernel<false, 4>), grid, dim3(256), 0, s, a);
  }
  return tw_prof_after(s);
}

extern "C" int twilight_int4_score_tokens(const twilight_kv_t* kv, const void* q, const int32_t* cand_tokens,
                                          const int32_t* cand_count, int32_t max_cand, float* scores, int32_t* dots,
                                          void* stream) {
  TwDims d;
  if (int e = tw_check_kv(kv, &d)) return e;
  if (!q || !scores || !cand_tokens || !cand_count || !kv->kq_pool || !kv->kq_meta) return TW_EINVAL;
  if (int e = tw_check_tokens(d, max_cand)) return e;
  return run_score_tokens(kv, d, q, cand_tokens, cand_count, max_cand, scores, dots, nullptr, (hipStream_t)stream);
}

extern "C" int twilight_topp_prune_tokens(const twilight_kv_t* kv, const void* q, const int32_t* cand_tokens,
                                          const int32_t* cand_count, int32_t max_cand, float p,
                                          int32_t* kept_count, int32_t* kept_idx, int32_t kept_stride,
                                          int32_t* union_count, int32_t* union_idx, int32_t union_stride,
                                          uint32_t* status, void* ws, size_t ws_bytes, void* stream) {
  TwDims d;
  if (int e = tw_check_kv(kv, &d)) return e;
  if (!q || !cand_tokens || !cand_count || !kept_count || !union_count || !union_idx || !status || !kv->kq_pool || !kv->kq_meta)
    return TW_EINVAL;
  if (!(p > 0.f) || p > 1.f || union_stride <= 0 || (kept_idx && kept_stride <= 0)) return TW_EINVAL;
  if (int e = tw_check_tokens(d, max_cand)) return e;
  const PruneWs L = tw_prune_layout_tokens(d, max_cand);
  if (!ws || ws_bytes < L.total) return TW_EWORKSPACE;
  hipStream_t s = (hipStream_t)stream;
  float* scores = (float*)((char*)ws + L.scores);
  uint32_t* arrive = (uint32_t*)((char*)ws + L.arrive);
  if (int e = run_score_tokens(kv, d, q, cand_tokens, cand_count, max_cand, scores, nullptr, arrive, s)) return e;
  HeadArgs f;
  f.scores = scores; f.sel_pages = cand_tokens; f.sel_count = cand_count; f.seq_lens = kv->seq_lens;
  f.kept_count = kept_count; f.kept_idx = kept_idx; f.bitmaps = (uint32_t*)((char*)ws + L.bitmaps); f.arrive = arrive;
  f.union_count = union_count; f.union_idx = union_idx; f.status = status;
  f.Hq = d.Hq; f.Hkv = d.Hkv; f.max_pages = d.max_pages; f.max_sel = max_cand; f.cand_stride = max_cand;
  f.kept_stride = kept_stride; f.words_stride = L.words_stride; f.union_stride = union_stride; f.p = p;
  f.q = nullptr; f.page_table = nullptr; f.kq_pool = nullptr; f.kq_meta = nullptr; f.pool_pages = 0;
  f.bounds = nullptr; f.budget = nullptr; f.sel_pages_w = nullptr; f.sel_count_w = nullptr;
  return launch_topp<true>(f, d, max_cand, s);
}
