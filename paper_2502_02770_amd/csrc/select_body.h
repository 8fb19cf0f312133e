// Selection of the Kp largest entries of one row of fp32 scores by a whole workgroup (Section 4.1: the page
// selector's top-k; also the channel-sparse token selector's).  Shared by the selection kernels and by the per-head
// pruner kernel that selects its pages itself.
#pragma once
#include "tw_common.h"

// Rows of up to SEL_LDS_MAX entries: keys staged in LDS.
// The Kp-th largest bound is located by bucketing the live key interval
// linearly into 2048 buckets (one pass when the bounds are spread out),
// narrowing to the bucket that holds it, and finishing with an exact rank
// computation once at most 256 candidates remain.
constexpr int SEL_LDS_PAGES = 8192;      // rows up to here run two workgroups per CU
constexpr int SEL_LDS_MAX = 32768;       // longest row whose keys fit in LDS (128 KiB of the CU's 160)
constexpr int SEL_NB = 2048;
constexpr int SEL_CAP = 256;


// entries of a sequence's row and how many of them the budget asks for (UNIT = tokens per entry: 16 or 1)
template <int UNIT>
__device__ __forceinline__ void tw_select_sizes(int n, int B, int max_pages, int max_sel, int* P_out, int* K_out) {
  int P = n > 0 ? (n + UNIT - 1) / UNIT : 0;
  if (P > max_pages) P = max_pages;
  long long kp = B > 0 ? ((long long)B + UNIT - 1) / UNIT : 0;
  if (kp > P) kp = P;
  if (kp > max_sel) kp = max_sel;
  *P_out = P;
  *K_out = (int)kp;
}

// The Kp (0 < Kp < P) largest of sc[0..P), ties to the lower index, written in ascending index order to out[0..Kp)
// (global) and, when given, to out_lds.  Called by all NT threads of the workgroup.  LDS of the caller: key_s[P],
// hist[SEL_NB], ck[SEL_CAP], ci[SEL_CAP].  SB: first phase-stamp slot (timing builds).
// EMAX > 0 (rows of at most EMAX * NT entries): thread t brings a value for each of the E entries [t * E, (t + 1) * E)
// it will list - pay[e] for entry t * E + e - which goes to pay_lds in list order for the selected ones; E =
// ceil(P / NT).  PRE: the caller asked for everything before it knew the row's length: E = EMAX, and pre[e] holds the
// score of entry e * NT + t (sc is then not read).
template <int NT, int SB, int EMAX = 0, bool PRE = false>
__device__ __forceinline__ void tw_select_row(const float* sc, int P, int Kp, int max_sel, int32_t* out, int32_t* out_lds,
                                              uint32_t* key_s, uint32_t* hist, uint32_t* ck, int32_t* ci,
                                              const int32_t* pay = nullptr, int32_t* pay_lds = nullptr,
                                              const float* pre = nullptr) {
  constexpr int NW = NT / 64, BPT = SEL_NB / NT;      // waves; histogram buckets per thread
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  TW_STAMP(SB);

  __shared__ uint32_t wsum[16];
  __shared__ uint32_t red_lo[NW], red_hi[NW];
  __shared__ uint32_t sh_bkt, sh_need, sh_pop, sh_n, sh_T, sh_need_eq;

  uint32_t lo = 0xFFFFFFFFu, hi = 0u;
  if (PRE) {
#pragma unroll
    for (int j = 0; j < (EMAX > 0 ? EMAX : 1); ++j) {
      const int i = j * NT + tid;
      if (i < P) {
        const uint32_t k = tw_float_key(pre[j]);
        key_s[i] = k;
        lo = k < lo ? k : lo;
        hi = k > hi ? k : hi;
      }
    }
  } else
  for (int base = 0; base < P; base += 8 * NT) {    // 8 clamped loads in flight per thread
    float v[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) { const int i = base + j * NT + tid; v[j] = sc[i < P ? i : P - 1]; }
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const int i = base + j * NT + tid;
      if (i < P) {
        const uint32_t k = tw_float_key(v[j]);
        key_s[i] = k;
        lo = k < lo ? k : lo;
        hi = k > hi ? k : hi;
      }
    }
  }
  lo = ~tw_wave_max_u32(~lo);
  hi = tw_wave_max_u32(hi);
  if (lane == 0) { red_lo[wave] = lo; red_hi[wave] = hi; }
  if (tid == 0) sh_n = 0;
  for (int i = tid; i < SEL_NB; i += NT) hist[i] = 0;     // for the first pass (cleared again before any later one)
  __syncthreads();
  uint32_t klo = red_lo[0], khi = red_hi[0];
#pragma unroll
  for (int w = 1; w < NW; ++w) { klo = red_lo[w] < klo ? red_lo[w] : klo; khi = red_hi[w] > khi ? red_hi[w] : khi; }

  uint32_t need = (uint32_t)Kp, T = 0, need_eq = 0;
  TW_STAMP(SB + 1);
#pragma unroll 1
  for (int pass = 0;; ++pass) {
    if (pass < 6) TW_STAMP(SB + 2 + pass);
    if (klo == khi) { T = klo; need_eq = need; break; }                    // everything left ties
    const float smn = tw_key_to_float(klo), smx = tw_key_to_float(khi);
    const float scale = (float)SEL_NB / (smx - smn);
    // Buckets are linear in the bound's value while that works: a finite scale over a normal span, and only
    // for the first passes.  Otherwise (spans in the subnormal range, infinite bounds, rows that keep falling
    // into one bucket) they are linear in the order-preserving key, which splits any span of at least 2048
    // keys 2048 ways and resolves a shorter one exactly, so every pass narrows the interval.
    const bool by_key = !(scale <= 3.0e38f) || !(smx - smn >= 1.1754944e-38f) || pass >= 3;
    const uint32_t span = khi - klo;
    const int kshift = span < (uint32_t)SEL_NB ? 0 : 32 - __clz(span) - 11;
    auto bucket_of = [&](uint32_t k) -> int {
      if (by_key) return (int)((k - klo) >> kshift);
      const int bk = (int)((tw_key_to_float(k) - smn) * scale);
      return bk > SEL_NB - 1 ? SEL_NB - 1 : (bk < 0 ? 0 : bk);
    };
    if (pass > 0) {
      for (int i = tid; i < SEL_NB; i += NT) hist[i] = 0;
      __syncthreads();
    }
    for (int i = tid; i < P; i += NT) {
      const uint32_t k = key_s[i];
      if (k >= klo && k <= khi) atomicAdd(&hist[bucket_of(k)], 1u);
    }
    __syncthreads();
    // thread t owns the BPT buckets below 2047 - BPT*t, walked downwards
    uint32_t c[BPT], mine = 0;
#pragma unroll
    for (int j = 0; j < BPT; ++j) { c[j] = hist[SEL_NB - 1 - (BPT * tid + j)]; mine += c[j]; }
    uint32_t total;
    const uint32_t incl = tw_block_scan_u32_open(mine, wsum, &total);   // (wsum is next written behind the barrier below)
    uint32_t above = incl - mine;
    if (above < need && incl >= need) {
#pragma unroll
      for (int j = 0; j < BPT; ++j) {
        if (above < need && above + c[j] >= need) { sh_bkt = SEL_NB - 1 - (BPT * tid + j); sh_need = need - above; sh_pop = c[j]; }
        above += c[j];
      }
    }
    __syncthreads();
    const int bkt = (int)sh_bkt;
    need = sh_need;
    const uint32_t pop = sh_pop;
    // narrow to the keys of that bucket; collect them when few enough for the exact finish
    const bool small = pop <= SEL_CAP && pop != need;
    uint32_t nlo = 0xFFFFFFFFu, nhi = 0u;
    for (int i = tid; i < P; i += NT) {
      const uint32_t k = key_s[i];
      if (k >= klo && k <= khi) {
        if (bucket_of(k) == bkt) {
          nlo = k < nlo ? k : nlo;
          nhi = k > nhi ? k : nhi;
          if (small) { const uint32_t at = atomicAdd(&sh_n, 1u); if (at < SEL_CAP) { ck[at] = k; ci[at] = i; } }
        }
      }
    }
    nlo = ~tw_wave_max_u32(~nlo);
    nhi = tw_wave_max_u32(nhi);
    if (lane == 0) { red_lo[wave] = nlo; red_hi[wave] = nhi; }
    __syncthreads();
    klo = red_lo[0]; khi = red_hi[0];
#pragma unroll
    for (int w = 1; w < NW; ++w) { klo = red_lo[w] < klo ? red_lo[w] : klo; khi = red_hi[w] > khi ? red_hi[w] : khi; }
    if (pop == need) { T = klo; need_eq = 0xFFFFFFFFu; break; }   // the whole bucket is taken
    if (small) {
      // exact: the candidate of rank need-1 (by bound, then by lower page id) is the last one taken
      if (tid < (int)pop) {
        const uint32_t kx = ck[tid];
        const int ix = ci[tid];
        uint32_t rank = 0, eq_lower = 0;
        for (uint32_t j = 0; j < pop; ++j) {
          const uint32_t kj = ck[j];
          const int ij = ci[j];
          rank += (kj > kx || (kj == kx && ij < ix)) ? 1u : 0u;
          eq_lower += (kj == kx && ij < ix) ? 1u : 0u;
        }
        if (rank == need - 1) { sh_T = kx; sh_need_eq = eq_lower + 1; }
      }
      __syncthreads();
      T = sh_T;
      need_eq = sh_need_eq;
      break;
    }
    __syncthreads();                              // red_* and hist are rewritten by the next pass
  }

  TW_STAMP(SB + 10);
  // ---- ordered emit: thread t owns the contiguous pages [t*E, (t+1)*E)
  const int E = PRE ? EMAX : (P + NT - 1) / NT;
  const int i0 = tid * E, i1 = (i0 + E < P) ? i0 + E : P;
  uint32_t gt = 0, eq = 0;
  for (int i = i0; i < i1; ++i) { const uint32_t k = key_s[i]; gt += k > T ? 1u : 0u; eq += k == T ? 1u : 0u; }
  uint32_t total;
  const uint32_t incl = tw_block_scan_u32_open(gt | (eq << 16), wsum, &total);   // (last use of wsum)
  uint32_t gt_before = (incl & 0xFFFFu) - gt, eq_before = (incl >> 16) - eq;
  if (EMAX > 0) {
#pragma unroll
    for (int e = 0; e < (EMAX > 0 ? EMAX : 1); ++e) {
      const int i = i0 + e;
      if (i < i1) {
        const uint32_t k = key_s[i];
        if (k > T || (k == T && eq_before < need_eq)) {
          const uint32_t pos = gt_before + (eq_before < need_eq ? eq_before : need_eq);
          if (pos < (uint32_t)max_sel) { out[pos] = i; out_lds[pos] = i; pay_lds[pos] = pay[e]; }
        }
        gt_before += k > T ? 1u : 0u;
        eq_before += k == T ? 1u : 0u;
      }
    }
  } else
  for (int i = i0; i < i1; ++i) {
    const uint32_t k = key_s[i];
    if (k > T || (k == T && eq_before < need_eq)) {
      const uint32_t pos = gt_before + (eq_before < need_eq ? eq_before : need_eq);
      if (pos < (uint32_t)max_sel) { out[pos] = i; if (out_lds) out_lds[pos] = i; }
    }
    gt_before += k > T ? 1u : 0u;
    eq_before += k == T ? 1u : 0u;
  }
  TW_STAMP(SB + 11);
}
