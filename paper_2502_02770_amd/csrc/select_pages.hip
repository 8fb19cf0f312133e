// Stage 1: Quest-style page selector (paper: Section 4.1 "Token Selector",
// Section 4 challenge C1: pooling per 16-token page).
//
// page_score:  U[h,P] = sum_d max(q_d*min[P,d], q_d*max[P,d]).  16 lanes per
//              page, each lane one 16-byte load of min and of max (8 dims);
//              the G query heads of the KV head share the loaded bounds.
//              fp32 order: 8 dims left to right per lane, then a pairwise
//              DPP tree over the 16 lanes (bit-reproducible).
// page_select: per (sequence, query head) the Kp largest bounds, ties to the
//              lower page id, by a 4 x 8-bit radix select on the order-
//              preserving key, then an ordered compaction (ascending ids).
//
// page_score<G, true> also appends the decode step's one new token per sequence on its way
// (twilight_append_select): the 16 lanes that own the page the token falls into store its K/V
// rows, quantise K, and fold it into the page's bounds before scoring them.
#include <atomic>
#include <stdlib.h>
#include "tw_common.h"
#include "kquant_common.h"
#include "topp_common.h"
#include "select_body.h"

namespace {

constexpr int PS_PAGES_PER_WG = 32;   // 4 waves x 4 pages x 2 iterations

struct ScoreArgs {
  const uint32_t* q;          // bf16 pairs [b][Hq][64]
  const uint4* page_minmax;   // [page][Hkv][2][16]
  const int32_t* page_table;
  const int32_t* seq_lens;
  float* scores;              // [b][Hq][max_pages]
  int Hq, Hkv, max_pages;
  long long pool_pages;
  // the step's new token (APPEND only): one row per sequence, [b][Hkv][128] bf16
  const uint4* k_new;
  const uint4* v_new;         // or nullptr
  const int32_t* new_pos;     // [b] position of the new token, < 0: none
  uint4* k_pool;              // or nullptr (no bf16 copy kept)
  uint4* v_pool;
  uint32_t* kq_pool;          // INT4 codes, 16 words per token
  uint32_t* kq_meta;
  uint4* page_minmax_w;
  uint32_t* arrive;           // [b][Hkv] arrival counters of a top-p launch that follows, cleared here, or nullptr
};

template <int G, bool APPEND, int BITS = 4>
__global__ __launch_bounds__(256) void page_score_kernel(ScoreArgs a) {
  // KV head fastest in dispatch order: the 8 heads' bounds of a pool page are 4 KiB contiguous,
  // and the workgroups that read them start next to each other
  const int b = blockIdx.z, g = blockIdx.x;
  const int tid = threadIdx.x, seg = tid & 15, grp = tid >> 4;   // grp: 0..15 page slot in the WG
  TW_STAMP(0);
  const int n = a.seq_lens[b];
  // last pages first: the workgroup that appends the step's new token (the sequence's last page) has the longest
  // chain of dependent accesses and should not be the one that starts last
  const int base = (int)(gridDim.y - 1 - blockIdx.y) * PS_PAGES_PER_WG;
  // page-table entries of this lane's 4 pages: issued before the sequence length is known (any entry of
  // the row may be read; entries beyond the last page are ignored below), so that the two loads overlap
  constexpr int IT = PS_PAGES_PER_WG / 16;
  long long pool[IT];
#pragma unroll
  for (int it = 0; it < IT; ++it) {
    const int lp = base + it * 16 + grp;
    pool[it] = a.page_table[(long long)b * a.max_pages + (lp < a.max_pages ? lp : a.max_pages - 1)];
  }
  int P = (n + TW_PAGE - 1) / TW_PAGE;
  if (P > a.max_pages) P = a.max_pages;
  // (the counters of a top-p launch that follows are cleared on the way out, after every load of the kernel: a store
  //  ahead of them would turn the scalar loads of the prologue into vector loads that wait for one another)
  const bool clears = a.arrive && blockIdx.y == 0 && tid == 0;
  if (base >= P) {
    if (clears) a.arrive[(b * a.Hkv + g) * TW_CTR] = 0;
    return;
  }

  // q of the G heads, the 8 dims of this lane; the sign decides which corner
  // of the [min,max] box maximises q_d * k_d.
  float q[G][8];
#pragma unroll
  for (int h = 0; h < G; ++h) {
    const uint4 r = *(const uint4*)(a.q + ((long long)(b * a.Hq + g * G + h)) * 64 + seg * 4);
    tw_unpack8(r, q[h]);
  }

  // then all 8 bound loads (clamped addresses, unconditional) so that they are in flight together;
  // unmapped pages are masked afterwards
  bool live[IT], ok[IT];
#pragma unroll
  for (int it = 0; it < IT; ++it) live[it] = base + it * 16 + grp < P;
  uint4 rmn[IT], rmx[IT];
#pragma unroll
  for (int it = 0; it < IT; ++it) {
    ok[it] = live[it] && pool[it] >= 0 && pool[it] < a.pool_pages;
    const uint4* pm = a.page_minmax + ((ok[it] ? pool[it] : 0) * a.Hkv + g) * 32;
    rmn[it] = tw_ld_stream(pm + seg);
    rmx[it] = tw_ld_stream(pm + 16 + seg);
  }
  if (APPEND) {
    // the page of the new token, if it lies in this workgroup's pages: its 16 owner lanes append
    const int sp = a.new_pos[b];
    const int off = (sp >> 4) - base;
    if (sp >= 0 && sp < n && off >= 0 && off < PS_PAGES_PER_WG && (off & 15) == grp) {
#pragma unroll
      for (int it = 0; it < IT; ++it) {
        if (it == (off >> 4) && ok[it]) {
          const long long row = (long long)b * a.Hkv + g;
          const uint4 raw = a.k_new[row * 16 + seg];
          const long long slot = (pool[it] * a.Hkv + g) * TW_PAGE + (sp & 15);
          if (a.k_pool) a.k_pool[slot * 16 + seg] = raw;
          if (a.v_new) a.v_pool[slot * 16 + seg] = a.v_new[row * 16 + seg];
          float x[8];
          tw_unpack8(raw, x);
          uint32_t word, word2, meta;
          tw_quantize_lane8<BITS>(x, seg, &word, &word2, &meta);
          if (BITS == 4) a.kq_pool[slot * 16 + seg] = word;
          else if (BITS == 8) ((uint2*)a.kq_pool)[slot * 16 + seg] = make_uint2(word, word2);
          else if ((seg & 1) == 0) a.kq_pool[slot * 8 + (seg >> 1)] = word;
          if ((seg & 3) == 0) a.kq_meta[slot * 4 + (seg >> 2)] = meta;
          // bounds: the token alone if it opens the page, else folded into the page's older tokens
          float mn[8], mx[8];
          tw_unpack8(rmn[it], mn);
          tw_unpack8(rmx[it], mx);
#pragma unroll
          for (int i = 0; i < 8; ++i) {
            mn[i] = (sp & 15) ? fminf(mn[i], x[i]) : x[i];
            mx[i] = (sp & 15) ? fmaxf(mx[i], x[i]) : x[i];
          }
          // min / max of bf16 values are bf16 values: the top 16 bits are exact
          uint4 wmn, wmx;
          wmn.x = (__float_as_uint(mn[0]) >> 16) | (__float_as_uint(mn[1]) & 0xFFFF0000u);
          wmn.y = (__float_as_uint(mn[2]) >> 16) | (__float_as_uint(mn[3]) & 0xFFFF0000u);
          wmn.z = (__float_as_uint(mn[4]) >> 16) | (__float_as_uint(mn[5]) & 0xFFFF0000u);
          wmn.w = (__float_as_uint(mn[6]) >> 16) | (__float_as_uint(mn[7]) & 0xFFFF0000u);
          wmx.x = (__float_as_uint(mx[0]) >> 16) | (__float_as_uint(mx[1]) & 0xFFFF0000u);
          wmx.y = (__float_as_uint(mx[2]) >> 16) | (__float_as_uint(mx[3]) & 0xFFFF0000u);
          wmx.z = (__float_as_uint(mx[4]) >> 16) | (__float_as_uint(mx[5]) & 0xFFFF0000u);
          wmx.w = (__float_as_uint(mx[6]) >> 16) | (__float_as_uint(mx[7]) & 0xFFFF0000u);
          uint4* pm = a.page_minmax_w + (pool[it] * a.Hkv + g) * 32;
          pm[seg] = wmn;
          pm[16 + seg] = wmx;
          rmn[it] = wmn;
          rmx[it] = wmx;
        }
      }
    }
  }
#pragma unroll
  for (int it = 0; it < IT; ++it) {
    const int lp = base + it * 16 + grp;
    float mn[8], mx[8];
    tw_unpack8(rmn[it], mn);
    tw_unpack8(rmx[it], mx);
    float part[G];
#pragma unroll
    for (int h = 0; h < G; ++h) {
      float acc = 0.f;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        // the product of two bf16 values is exact in fp32, so this fused
        // multiply-add rounds exactly like "acc + q*v"
        const float v = q[h][i] > 0.f ? mx[i] : mn[i];
        acc = __builtin_fmaf(q[h][i], v, acc);
      }
      part[h] = acc;
    }
    if constexpr (G >= 4) {
      // The pairwise tree over the 16 lanes (l^1, l^2, l^4, l^8) for four heads at once: at the first two levels a
      // lane keeps the half of its values that one bit of its lane id selects and adds the partner's copy of them
      // (the same two operands as the plain tree adds, so the same sums), which leaves lane l with the quad sum of
      // head 2 * (l & 1) + ((l >> 1) & 1); the last two levels rotate the row by 4 and by 8 (a lane reads lane
      // l - 4, then l - 8, modulo 16), which for lanes 4..7 are exactly l ^ 4 and l ^ 8 of the same head.  Lanes 4..7
      // end with the four totals: 5 additions and 6 selects per four heads instead of 16 additions.
      const bool b0 = seg & 1, b1 = seg & 2;
#pragma unroll
      for (int h4 = 0; h4 < G; h4 += 4) {
        const float k0 = b0 ? part[h4 + 2] : part[h4 + 0], s0 = b0 ? part[h4 + 0] : part[h4 + 2];
        const float k1 = b0 ? part[h4 + 3] : part[h4 + 1], s1 = b0 ? part[h4 + 1] : part[h4 + 3];
        const float a0 = __fadd_rn(k0, tw_dpp_f<TW_DPP_XOR1>(s0));     // head h4 + 2 * b0
        const float a1 = __fadd_rn(k1, tw_dpp_f<TW_DPP_XOR1>(s1));     // head h4 + 2 * b0 + 1
        const float kk = b1 ? a1 : a0, ss = b1 ? a0 : a1;
        float t = __fadd_rn(kk, tw_dpp_f<TW_DPP_XOR2>(ss));            // head h4 + 2 * b0 + b1, summed over the quad
        t = __fadd_rn(t, tw_dpp_f<0x124>(t));                          // row_ror:4 - lanes 4..7 and 12..15 read l ^ 4
        t = __fadd_rn(t, tw_dpp_f<0x128>(t));                          // row_ror:8 - every lane reads l ^ 8
        if ((seg >> 2) == 1 && live[it])
          a.scores[((long long)(b * a.Hq + g * G + h4 + 2 * (seg & 1) + ((seg >> 1) & 1))) * a.max_pages + lp] =
              ok[it] ? __fadd_rn(t, 0.0f) : -3.402823466e38f;          // unmapped page: ranks last
      }
    } else {
#pragma unroll
      for (int h = 0; h < G; ++h) {
        const float acc = tw_row16_sum(part[h]);
        if (seg == 0 && live[it])
          a.scores[((long long)(b * a.Hq + g * G + h)) * a.max_pages + lp] =
              ok[it] ? __fadd_rn(acc, 0.0f) : -3.402823466e38f;   // unmapped page: ranks last
      }
    }
  }
  if (clears) a.arrive[(b * a.Hkv + g) * TW_CTR] = 0;
}

struct SelectArgs {
  const float* scores;        // [b][Hq][max_pages]
  const int32_t* seq_lens;
  const int32_t* budget;
  int32_t* sel_pages;         // [b][Hq][max_sel]
  int32_t* sel_count;
  int Hq, max_pages, max_sel;
  int p_above, p_upto;        // the LDS kernel takes the heads with p_above < pages <= p_upto
};
// The kernels' UNIT parameter = tokens per row entry: 16 = pages (budget and lengths are in tokens), 1 = the rows hold one
// score per token (channel-sparse token selector; max_pages is then the row length in tokens).

template <int UNIT>
__device__ __forceinline__ void tw_select_sizes(const SelectArgs& a, int n, int B, int* P_out, int* K_out) {
  ::tw_select_sizes<UNIT>(n, B, a.max_pages, a.max_sel, P_out, K_out);
}

template <int UNIT>
__global__ __launch_bounds__(256) void page_select_kernel(SelectArgs a) {
  const int b = blockIdx.y, h = blockIdx.x, tid = threadIdx.x;
  int P, Kp;
  tw_select_sizes<UNIT>(a, a.seq_lens[b], a.budget[b], &P, &Kp);
  const float* sc = a.scores + ((long long)(b * a.Hq + h)) * a.max_pages;
  int32_t* out = a.sel_pages + ((long long)(b * a.Hq + h)) * a.max_sel;
  if (tid == 0) a.sel_count[b * a.Hq + h] = Kp;
  if (Kp == 0) return;
  if (Kp == P) {                         // budget covers the sequence: every page
    for (int i = tid; i < P; i += 256) out[i] = i;
    return;
  }

  __shared__ uint32_t hist[256];
  __shared__ uint32_t wsum[17];
  __shared__ uint32_t sh_prefix, sh_remaining;
  uint32_t prefix = 0, remaining = (uint32_t)Kp;
  // radix select of the Kp-th largest key, 8 bits per pass from the top
#pragma unroll 1
  for (int shift = 24; shift >= 0; shift -= 8) {
    hist[tid] = 0;
    __syncthreads();
    const uint32_t himask = shift == 24 ? 0u : (0xFFFFFFFFu << (shift + 8));
    for (int i = tid; i < P; i += 256) {
      const uint32_t key = tw_float_key(sc[i]);
      if ((key & himask) == prefix) atomicAdd(&hist[(key >> shift) & 255u], 1u);
    }
    __syncthreads();
    // thread t looks at digit 255-t: inclusive count of keys with digit >= its own
    const uint32_t mine = hist[255 - tid];
    uint32_t total;
    const uint32_t incl = tw_block_scan_u32(mine, wsum, &total);
    if (incl >= remaining && incl - mine < remaining) {
      sh_prefix = prefix | ((uint32_t)(255 - tid) << shift);
      sh_remaining = remaining - (incl - mine);
    }
    __syncthreads();
    prefix = sh_prefix;
    remaining = sh_remaining;
    __syncthreads();
  }
  // prefix = key of the Kp-th largest bound; `remaining` pages with exactly
  // that key are taken, lowest ids first.
  const uint32_t T = prefix, need_eq = remaining;
  uint32_t run_gt = 0, run_eq = 0;
#pragma unroll 1
  for (int base = 0; base < P; base += 256) {
    const int i = base + tid;
    uint32_t key = 0;
    const bool in = i < P;
    if (in) key = tw_float_key(sc[i]);
    const uint32_t fgt = (in && key > T) ? 1u : 0u;
    const uint32_t feq = (in && key == T) ? 1u : 0u;
    uint32_t total;
    const uint32_t incl = tw_block_scan_u32(fgt | (feq << 16), wsum, &total);
    const uint32_t gt_before = run_gt + (incl & 0xFFFFu) - fgt;
    const uint32_t eq_before = run_eq + (incl >> 16) - feq;
    if (fgt || (feq && eq_before < need_eq)) {
      const uint32_t pos = gt_before + (eq_before < need_eq ? eq_before : need_eq);
      if (pos < (uint32_t)a.max_sel) out[pos] = i;
    }
    run_gt += total & 0xFFFFu;
    run_eq += total >> 16;
  }
}


template <int NT, int UNIT>
__global__ __launch_bounds__(NT) void page_select_lds_kernel(SelectArgs a) {
  const int b = blockIdx.y, h = blockIdx.x, tid = threadIdx.x;
  int P, Kp;
  tw_select_sizes<UNIT>(a, a.seq_lens[b], a.budget[b], &P, &Kp);
  if (P <= a.p_above || P > a.p_upto) return;     // another launch's head (block-uniform)
  const float* sc = a.scores + ((long long)(b * a.Hq + h)) * a.max_pages;
  int32_t* out = a.sel_pages + ((long long)(b * a.Hq + h)) * a.max_sel;
  if (tid == 0) a.sel_count[b * a.Hq + h] = Kp;
  if (Kp == 0) return;
  if (Kp == P) {
    for (int i = tid; i < P; i += NT) out[i] = i;
    return;
  }
  extern __shared__ uint32_t key_s[];             // one key per row entry (the launch sizes it to the row bound)
  __shared__ uint32_t hist[SEL_NB];
  __shared__ uint32_t ck[SEL_CAP];
  __shared__ int32_t ci[SEL_CAP];
  tw_select_row<NT, 10>(sc, P, Kp, a.max_sel, out, nullptr, key_s, hist, ck, ci);
}

template <int G>
void launch_score(const ScoreArgs& a, dim3 grid, bool append, int bits, hipStream_t s) {
  if (!append)        TW_LAUNCH((page_score_kernel<G, false>), grid, dim3(256), 0, s, a);
  else if (bits == 4) TW_LAUNCH((page_score_kernel<G, true, 4>), grid, dim3(256), 0, s, a);
  else if (bits == 8) TW_LAUNCH((page_score_kernel<G, true, 8>), grid, dim3(256), 0, s, a);
  else                TW_LAUNCH((page_score_kernel<G, true, 2>), grid, dim3(256), 0, s, a);
}

}  // namespace

#ifdef TW_PHASE_TIMING
extern "C" int twilight_debug_stamps_select(unsigned long long* host_out) {
  return hipMemcpyFromSymbol(host_out, HIP_SYMBOL(tw_dbg_stamps), sizeof(unsigned long long) * 64) == hipSuccess ? 0 : -1;
}
#endif

// Rows of more than 12288 entries need more dynamic LDS than a launch may ask for by default: raised once per device.
template <int UNIT>
static bool select_lds_big_ok() {
  static std::atomic<int> done[TW_MAX_DEVICES];   // 0 = not tried, 1 = ok, 2 = refused
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= TW_MAX_DEVICES) return false;
  int st = done[dev].load(std::memory_order_relaxed);
  if (st == 0) {
    const hipError_t e = hipFuncSetAttribute((const void*)page_select_lds_kernel<1024, UNIT>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                             SEL_LDS_MAX * 4);
    if (e != hipSuccess) (void)hipGetLastError();
    st = e == hipSuccess ? 1 : 2;
    done[dev].store(st, std::memory_order_relaxed);
  }
  return st == 1;
}

// The selection kernels by row length (entries per row = sa.max_pages) and number of heads.
template <int UNIT>
static int launch_select(SelectArgs sa, const TwDims& d, hipStream_t s) {
  const int L = sa.max_pages;
  sa.p_above = -1; sa.p_upto = L;
  // Many heads and rows of up to 8192 entries (ragged batches): the 1024-thread kernel fits two
  // workgroups per CU; rows of at most 2048 entries go to a 256-thread launch of their own.
  if (L > 2048 && L <= SEL_LDS_PAGES && (long long)d.batch * d.Hq > 2ll * tw_num_cus()) {
    sa.p_upto = 2048;
    tw_prof_before(TW_K_PAGE_SELECT, s);
    TW_LAUNCH((page_select_lds_kernel<256, UNIT>), dim3(d.Hq, d.batch), dim3(256), 2048 * 4, s, sa);
    if (int e = tw_prof_after(s)) return e;
    sa.p_above = 2048; sa.p_upto = L;
  }
  tw_prof_before(TW_K_PAGE_SELECT, s);
  // rows of 513..2048 entries: with few heads (at most two workgroups per CU) the 1024-thread variant is the
  // quicker one (6.7 against 8.4 us at 8 x 32 heads x 2048 pages); many heads are better served by small workgroups
  const bool few_heads = (long long)d.batch * d.Hq <= 2ll * tw_num_cus();
  if (L <= 512 || (L <= 2048 && !few_heads))
    TW_LAUNCH((page_select_lds_kernel<256, UNIT>), dim3(d.Hq, d.batch), dim3(256), (size_t)L * 4, s, sa);
  else if (L <= SEL_LDS_MAX && ((size_t)L * 4 <= 48 * 1024 || select_lds_big_ok<UNIT>()))
    TW_LAUNCH((page_select_lds_kernel<1024, UNIT>), dim3(d.Hq, d.batch), dim3(1024), (size_t)L * 4, s, sa);
  else
    TW_LAUNCH(page_select_kernel<UNIT>, dim3(d.Hq, d.batch), dim3(256), 0, s, sa);
  return tw_prof_after(s);
}

static int select_impl(const twilight_kv_t* kv, const void* q, const int32_t* budget_tokens,
                       int32_t* sel_pages, int32_t* sel_count, int32_t max_sel,
                       void* ws, size_t ws_bytes, void* stream,
                       bool append, const void* k_new, const void* v_new, const int32_t* new_pos,
                       uint32_t* arrive = nullptr, bool bounds_only = false) {
  TwDims d;
  if (int e = tw_check_kv(kv, &d)) return e;
  if (!q || !budget_tokens || !sel_pages || !sel_count || max_sel <= 0 || !kv->page_minmax) return TW_EINVAL;
  if (append) {
    if (!k_new || !new_pos || !kv->kq_pool || !kv->kq_meta) return TW_EINVAL;
    if (v_new && !kv->v_pool) return TW_EINVAL;
  }
  if (!ws || ws_bytes < twilight_workspace_bytes(TW_WS_SELECT, kv, max_sel, 0)) return TW_EWORKSPACE;
  hipStream_t s = (hipStream_t)stream;

  ScoreArgs a;
  a.q = (const uint32_t*)q; a.page_minmax = (const uint4*)kv->page_minmax;
  a.page_table = kv->page_table; a.seq_lens = kv->seq_lens; a.scores = (float*)ws;
  a.Hq = d.Hq; a.Hkv = d.Hkv; a.max_pages = d.max_pages; a.pool_pages = d.pool_pages;
  a.k_new = (const uint4*)k_new; a.v_new = (const uint4*)v_new; a.new_pos = new_pos;
  a.k_pool = (uint4*)kv->k_pool; a.v_pool = (uint4*)kv->v_pool;
  a.kq_pool = (uint32_t*)kv->kq_pool; a.kq_meta = (uint32_t*)kv->kq_meta;
  a.page_minmax_w = (uint4*)kv->page_minmax;
  a.arrive = arrive;
  dim3 grid(d.Hkv, (d.max_pages + PS_PAGES_PER_WG - 1) / PS_PAGES_PER_WG, d.batch);
  tw_prof_before(TW_K_PAGE_SCORE, s);
  switch (d.G) {
    case 1: launch_score<1>(a, grid, append, d.bits, s); break;
    case 2: launch_score<2>(a, grid, append, d.bits, s); break;
    case 4: launch_score<4>(a, grid, append, d.bits, s); break;
    default: launch_score<8>(a, grid, append, d.bits, s); break;
  }
  if (int e = tw_prof_after(s)) return e;
  if (bounds_only) return TW_OK;

  SelectArgs sa;
  sa.scores = (const float*)ws; sa.seq_lens = kv->seq_lens; sa.budget = budget_tokens;
  sa.sel_pages = sel_pages; sa.sel_count = sel_count;
  sa.Hq = d.Hq; sa.max_pages = d.max_pages; sa.max_sel = max_sel;
  return launch_select<TW_PAGE>(sa, d, s);
}

// Channel-sparse token selector (a Double-Sparsity-style base algorithm in front of the pruner; Section 4.1's
// black-box token selector, Sections 4.3 / 5): every token of a sequence is scored from the INT4 copy of K with the
// query restricted to the KV head's channel set, and the budget's worth of tokens with the largest estimate is handed
// over as a token list (ties to the lower position, ascending).
extern "C" int twilight_ds_select_tokens(const twilight_kv_t* kv, const void* q, const uint32_t* channel_mask,
                                         const int32_t* budget_tokens, int32_t* cand_tokens, int32_t* cand_count,
                                         int32_t max_cand, void* ws, size_t ws_bytes, void* stream) {
  TwDims d;
  if (int e = tw_check_kv(kv, &d)) return e;
  if (!q || !channel_mask || !budget_tokens || !cand_tokens || !cand_count || max_cand <= 0 || !kv->kq_pool || !kv->kq_meta)
    return TW_EINVAL;
  if ((long long)d.max_pages * TW_PAGE > 0x7FFFFFFFll / 4) return TW_EINVAL;
  if (!ws || ws_bytes < twilight_workspace_bytes(TW_WS_DS_SELECT, kv, max_cand, 0)) return TW_EWORKSPACE;
  hipStream_t s = (hipStream_t)stream;
  if (int e = tw_score_all_tokens_masked(kv, d, q, channel_mask, (float*)ws, s)) return e;
  SelectArgs sa;
  sa.scores = (const float*)ws; sa.seq_lens = kv->seq_lens; sa.budget = budget_tokens;
  sa.sel_pages = cand_tokens; sa.sel_count = cand_count;
  sa.Hq = d.Hq; sa.max_pages = d.max_pages * TW_PAGE; sa.max_sel = max_cand;
  return launch_select<1>(sa, d, s);
}

extern "C" int twilight_select_pages(const twilight_kv_t* kv, const void* q, const int32_t* budget_tokens,
                                     int32_t* sel_pages, int32_t* sel_count, int32_t max_sel,
                                     void* ws, size_t ws_bytes, void* stream) {
  return select_impl(kv, q, budget_tokens, sel_pages, sel_count, max_sel, ws, ws_bytes, stream, false, nullptr, nullptr, nullptr);
}

// ---- the selector for callers that must not allocate: same kernels, the bound scores go to a
// fixed array of device memory that the library's code object carries.  The array's name is only a
// host-side handle; its address on the current device comes from hipGetSymbolAddress, once per device.
static __device__ __align__(256) unsigned char scratch[TW_STATIC_SELECT_WS_BYTES];

static int static_scratch_ptr(void** out) {
  static std::atomic<void*> ptrs[TW_MAX_DEVICES];
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= TW_MAX_DEVICES) return TW_ELAUNCH;
  void* p = ptrs[dev].load(std::memory_order_acquire);
  if (!p) {
    // every GPU holds its own copy of the array at its own address; racing first calls look up the same value
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
      (void)hipGetLastError();
      return TW_ELAUNCH;
    }
    ptrs[dev].store(p, std::memory_order_release);
  }
  *out = p;
  return TW_OK;
}

extern "C" int twilight_select_pages_static(const twilight_kv_t* kv, const void* q, const int32_t* budget_tokens,
                                            int32_t* sel_pages, int32_t* sel_count, int32_t max_sel, void* stream) {
  TwDims d;
  if (int e = tw_check_kv(kv, &d)) return e;
  if (max_sel <= 0) return TW_EINVAL;
  const size_t need = twilight_workspace_bytes(TW_WS_SELECT, kv, max_sel, 0);
  if (need == 0) return TW_EINVAL;
  if (need > (size_t)TW_STATIC_SELECT_WS_BYTES) return TW_ELIMIT;
  void* ws = nullptr;
  if (int e = static_scratch_ptr(&ws)) return e;
  // every score the select kernels read is written by page_score in this call: nothing has to start at zero
  return select_impl(kv, q, budget_tokens, sel_pages, sel_count, max_sel, ws, need, stream, false, nullptr, nullptr, nullptr);
}

extern "C" int twilight_append_select(const twilight_kv_t* kv, const void* k_new, const void* v_new, const int32_t* new_pos,
                                      const void* q, const int32_t* budget_tokens,
                                      int32_t* sel_pages, int32_t* sel_count, int32_t max_sel,
                                      void* ws, size_t ws_bytes, void* stream) {
  return select_impl(kv, q, budget_tokens, sel_pages, sel_count, max_sel, ws, ws_bytes, stream, true, k_new, v_new, new_pos);
}

// Selector and pruner in one call (Section 4.1's pipeline up to the pruned index sets): page bounds (with the step's
// new token appended on the way when k_new is given), then - where the lists are short enough for one workgroup per
// head - a single launch that picks each head's pages, scores their tokens from the 4-bit copy of K, runs top-p and
// builds the group's union; otherwise the launches of twilight_select_pages and twilight_topp_prune.
extern "C" int twilight_select_prune(const twilight_kv_t* kv, const void* k_new, const void* v_new, const int32_t* new_pos,
                                     const void* q, const int32_t* budget_tokens, float p,
                                     int32_t* sel_pages, int32_t* sel_count, int32_t max_sel,
                                     int32_t* kept_count, int32_t* kept_idx, int32_t kept_stride,
                                     int32_t* union_count, int32_t* union_idx, int32_t union_stride,
                                     uint32_t* status, void* ws, size_t ws_bytes, void* stream) {
  TwDims d;
  if (int e = tw_check_kv(kv, &d)) return e;
  if (!q || !budget_tokens || !sel_pages || !sel_count || !kept_count || !union_count || !union_idx || !status ||
      !kv->kq_pool || !kv->kq_meta || max_sel <= 0) return TW_EINVAL;
  if (!(p > 0.f) || p > 1.f || union_stride <= 0 || (kept_idx && kept_stride <= 0)) return TW_EINVAL;
  if ((long long)max_sel * TW_PAGE > (1ll << 22)) return TW_EINVAL;
  const size_t sel_bytes = twilight_workspace_bytes(TW_WS_SELECT, kv, max_sel, 0);
  const size_t need = twilight_workspace_bytes(TW_WS_SELECT_PRUNE, kv, max_sel, 0);
  if (!ws || need == 0 || ws_bytes < need) return TW_EWORKSPACE;
  void* ws_prune = (char*)ws + sel_bytes;
  const bool append = k_new != nullptr;
  // 2: selection and scoring inside the top-p kernel, 1: scoring only, 0: the separate launches
  const int can = tw_prune_fused_ok(d, max_sel, true) ? 2 : (tw_prune_fused_ok(d, max_sel, false) ? 1 : 0);
  int mode = can;
  // few heads with long lists (a single long sequence): one workgroup per head cannot pull its list fast enough, the
  // scoring launch's many workgroups can (32 heads x 8192 candidates: 51.8 us per step separately, 56.0 us fused)
  if (max_sel * TW_PAGE > 4096 && (long long)d.batch * d.Hq < tw_num_cus()) mode = 0;
#ifdef TW_TUNING
  if (const char* e = getenv("TW_FUSE")) { const int m = atoi(e); mode = m < can ? m : can; }
#endif
  if (mode == 0) {
    if (int e = select_impl(kv, q, budget_tokens, sel_pages, sel_count, max_sel, ws, sel_bytes, stream, append, k_new, v_new,
                            new_pos)) return e;
    return twilight_topp_prune(kv, q, sel_pages, sel_count, max_sel, p, kept_count, kept_idx, kept_stride, union_count,
                               union_idx, union_stride, status, ws_prune, ws_bytes - sel_bytes, stream);
  }
  uint32_t* arrive = (uint32_t*)((char*)ws_prune + tw_prune_layout(d, max_sel, false).arrive);
  if (int e = select_impl(kv, q, budget_tokens, sel_pages, sel_count, max_sel, ws, sel_bytes, stream, append, k_new, v_new,
                          new_pos, arrive, mode == 2)) return e;
  return tw_prune_fused(kv, d, q, mode == 2 ? (const float*)ws : nullptr, budget_tokens, sel_pages, sel_count, max_sel, p,
                        kept_count, kept_idx, kept_stride, union_count, union_idx, union_stride, status, ws_prune,
                        (hipStream_t)stream);
}
