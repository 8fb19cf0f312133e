// Stage 3: variable-budget sparse decode attention over the paged bf16 KV
// cache (paper: Definition 3.1 restricted to the kept set and renormalised
// over it; Appendix B.2: every query head of a KV head attends over the
// group's union, the group-wise variable-length form; Section 4.2 load balancing: the
// (sequence, KV head) lists are flattened into equal-sized work items).
//
// Work item = (group, chunk of `chunk` consecutive list entries).  A
// persistent grid walks the items with a fixed stride; the item -> (group,
// chunk) map is a prefix sum over the groups' chunk counts that every
// workgroup rebuilds in LDS from the device-side list lengths, so no host
// round trip and no extra launch is needed.  Inside an item 16 lanes own one
// token row (a 16-byte load of K and of V each, 8 dims), the G query heads
// of the group share every loaded row, and each 16-lane row keeps its own
// online-softmax state; states are merged by log-sum-exp, first inside the
// workgroup, then across items by the combine kernel.
//
// The same kernel serves the per-head variant (the head-wise form of Appendix
// B.2): one list per query head, G = 1, list l reads KV head l / group size.
#include <stdlib.h>
#include <atomic>
#include "tw_common.h"

namespace {

constexpr float kLog2eRsqrtD = 0x1.0527dcp-3f;   // fp32(log2(e) / sqrt(128))
constexpr float kLn2 = 0x1.62e43p-1f;
constexpr float kNegBig = -1.0e30f;              // finite stand-in for -inf in running maxima
constexpr int DEC_MAX_CHUNK = 512;
constexpr unsigned DEC_ITEMS_PER_WG = 3;         // measured: 64-entry items at 1.2 per workgroup, 128 at 2.5, 256 at 2 were the best choices

struct DecodeArgs {
  const uint4* q;             // bf16 [b][Hq][16 x uint4]
  const uint4* k_pool;        // 16 uint4 per token row
  const uint4* v_pool;
  const int32_t* page_table;
  const int32_t* seq_lens;
  const int32_t* union_count; // or nullptr (dense)
  const int32_t* union_idx;   // or nullptr (dense)
  uint4* out;                 // bf16 [b][Hq][16 x uint4]
  float* lse;                 // or nullptr
  int32_t* ws_prefix;         // [NG + 1]
  float2* ws_ml;              // [items][G]
  float4* ws_acc;             // [items][G][32 x float4]
  int Hq, Hkv, max_pages, union_stride, NG, chunk;
  int fix_chunk;              // tuning: use `chunk` as given
  int LH, kv_div;             // lists per sequence (Hkv, or Hq with one list per query head); list l reads KV head l / kv_div
  long long pool_pages;
};

__device__ __forceinline__ float tw_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// row_newbcast:k - lane k of each row of 16 to all lanes of the row
template <int K>
__device__ __forceinline__ float tw_row_bcast(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x150 + K, 0xF, 0xF, false));
}
#define TW_DPP_ROR4 0x124
#define TW_DPP_ROR8 0x128

typedef __bf16 tw_bf16x2 __attribute__((ext_vector_type(2)));
// a.lo * b.lo + a.hi * b.hi + c on bf16 pairs (v_dot2c_f32_bf16)
__device__ __forceinline__ float tw_dot2_bf16(uint32_t a, uint32_t b, float c) {
  return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(tw_bf16x2, a), __builtin_bit_cast(tw_bf16x2, b), c, false);
}

template <int G>
__global__ __launch_bounds__(256, G == 4 ? 4 : 1) void sparse_decode_kernel(DecodeArgs a) {
  constexpr int R = (G + 3) / 4;                 // score values a lane ends up owning per sub-block
  constexpr int HB = G < 4 ? G : 4;              // heads merged through LDS at a time
  extern __shared__ int32_t prefix[];            // [NG + 1]
  __shared__ uint32_t wsum[16];
  __shared__ uint32_t red3[3][4];
  __shared__ int32_t rows[DEC_MAX_CHUNK];
  __shared__ float smax[2][4][8];                // [buffer][wave][head]
  __shared__ float4 macc[16][HB][32];            // per 16-lane row: accumulators of HB heads
  __shared__ float ml_s[16][8];                  // per row: softmax denominators
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, seg = tid & 15, rg = tid >> 4;
  const bool dense = a.union_idx == nullptr;
  const bool b3 = seg & 8, b2 = seg & 4, b1 = seg & 2, b0 = seg & 1;
  const int my_t = seg >> 2, my_hc = seg & 3;
  TW_STAMP(0);

  // ---- chunk length: the shortest of {c0, 2c0, 4c0} (<= 512) that leaves a workgroup at most
  //      DEC_ITEMS_PER_WG items, so that short lists are spread over all workgroups (whose phases then
  //      interleave) and long ones amortise the per-item set-up and merge
  uint32_t n0 = 0, n1 = 0, n2 = 0;
  const int c0 = a.chunk;
  for (int gi = tid; gi < a.NG; gi += 256) {
    int cnt;
    if (dense) { cnt = a.seq_lens[gi / a.LH]; if (cnt > a.max_pages * TW_PAGE) cnt = a.max_pages * TW_PAGE; }
    else { cnt = a.union_count[gi]; if (cnt > a.union_stride) cnt = a.union_stride; }
    if (cnt < 0) cnt = 0;
    n0 += (cnt + c0 - 1) / c0; n1 += (cnt + 2 * c0 - 1) / (2 * c0); n2 += (cnt + 4 * c0 - 1) / (4 * c0);
  }
  n0 = tw_wave_scan_u32(n0); n1 = tw_wave_scan_u32(n1); n2 = tw_wave_scan_u32(n2);
  if (lane == 63) { red3[0][wave] = n0; red3[1][wave] = n1; red3[2][wave] = n2; }
  __syncthreads();
  n0 = red3[0][0] + red3[0][1] + red3[0][2] + red3[0][3];
  n1 = red3[1][0] + red3[1][1] + red3[1][2] + red3[1][3];
  int chunk = c0;
  if (!a.fix_chunk && n0 > DEC_ITEMS_PER_WG * gridDim.x && 2 * c0 <= DEC_MAX_CHUNK) {
    chunk = 2 * c0;
    if (n1 > DEC_ITEMS_PER_WG * gridDim.x && 4 * c0 <= DEC_MAX_CHUNK) chunk = 4 * c0;
  }

  // ---- item map: exclusive prefix of per-group chunk counts
  uint32_t run = 0;
  for (int base = 0; base < a.NG; base += 256) {
    const int gi = base + tid;
    uint32_t c = 0;
    if (gi < a.NG) {
      int cnt;
      if (dense) { cnt = a.seq_lens[gi / a.LH]; if (cnt > a.max_pages * TW_PAGE) cnt = a.max_pages * TW_PAGE; }
      else { cnt = a.union_count[gi]; if (cnt > a.union_stride) cnt = a.union_stride; }
      if (cnt < 0) cnt = 0;
      c = (uint32_t)((cnt + chunk - 1) / chunk);
    }
    uint32_t total;
    const uint32_t incl = tw_block_scan_u32(c, wsum, &total);
    if (gi < a.NG) prefix[gi] = (int32_t)(run + incl - c);
    run += total;
  }
  if (tid == 0) prefix[a.NG] = (int32_t)run;
  __syncthreads();
  const int total_items = (int)run;
  TW_STAMP(1);
  if (blockIdx.x == 0)
    for (int i = tid; i <= a.NG; i += 256) a.ws_prefix[i] = prefix[i];

#pragma unroll 1
  for (int item = blockIdx.x; item < total_items; item += gridDim.x) {
    // group of this item: last gi with prefix[gi] <= item
    int lo = 0, hi = a.NG;
    while (hi - lo > 1) { const int mid = (lo + hi) >> 1; if (prefix[mid] <= item) lo = mid; else hi = mid; }
    const int gi = lo, b = gi / a.LH, l = gi % a.LH, g = l / a.kv_div;   // list l of sequence b, KV head g
    const int ck = item - prefix[gi];
    const int nchunks = prefix[gi + 1] - prefix[gi];
    // Everything the row staging reads that does not depend on another load goes out together: the sequence's
    // length, the list's length, this thread's (at most two) list entries - any entry of the list's row may be read,
    // those at or beyond the count are ignored below - and q.  The page-table entries then depend on the list
    // entries, the K/V rows on those: three round trips to memory per item instead of five.
    const int t0 = ck * chunk;
    // (dense: the same loads from an address that is always valid, their values unused - no branch between the loads)
    int nseq = a.seq_lens[b];                    // list entries at or beyond the sequence's end are ignored
    const int32_t* const cnt_p = dense ? a.seq_lens + b : a.union_count + gi;
    int cnt = *cnt_p;
    int tokv[DEC_MAX_CHUNK / 256];
#pragma unroll
    for (int j = 0; j < DEC_MAX_CHUNK / 256; ++j) {
      const int e = t0 + j * 256 + tid;
      const int32_t* const tp = dense ? a.seq_lens + b
                                      : a.union_idx + (long long)gi * a.union_stride + (e < a.union_stride ? e : a.union_stride - 1);
      const int tv = *tp;
      tokv[j] = dense ? e : tv;
    }
    // q of the G heads, this lane's 8 dims, as loaded (bf16 pairs)
    uint4 q[G];
#pragma unroll
    for (int h = 0; h < G; ++h) q[h] = a.q[((long long)(b * a.Hq + l * G + h)) * 16 + seg];
    // (keeps the list-entry loads up here: the compiler would otherwise move them down to their first use, behind
    //  the wait for the two lengths)
#pragma unroll
    for (int j = 0; j < DEC_MAX_CHUNK / 256; ++j) asm volatile("" : "+v"(tokv[j]));
    if (nseq > a.max_pages * TW_PAGE) nseq = a.max_pages * TW_PAGE;
    if (dense) cnt = nseq;
    else if (cnt > a.union_stride) cnt = a.union_stride;
    const int len = cnt - t0 < chunk ? cnt - t0 : chunk;

    // ---- stage the chunk's token rows (pool row ids) in LDS
#pragma unroll
    for (int j = 0; j < DEC_MAX_CHUNK / 256; ++j) {
      const int i = j * 256 + tid;
      if (i < chunk) {                            // block-uniform per j
        int r = -1;
        const int tok = tokv[j];
        if (i < len && tok >= 0 && tok < nseq) {
          const long long pp = a.page_table[(long long)b * a.max_pages + (tok >> 4)];
          if (pp >= 0 && pp < a.pool_pages) r = (int)((pp * a.Hkv + g) * TW_PAGE + (tok & 15));
        }
        rows[i] = r;
      }
    }
    if (item == 0) TW_STAMP(2);
    float acc[G][8], M[G], Mmine[R], lacc[R];
#pragma unroll
    for (int h = 0; h < G; ++h) {
      M[h] = kNegBig;
#pragma unroll
      for (int i = 0; i < 8; ++i) acc[h][i] = 0.f;
    }
#pragma unroll
    for (int r = 0; r < R; ++r) { Mmine[r] = kNegBig; lacc[r] = 0.f; }
    __syncthreads();

    const int nsub = (len + 63) >> 6;
#pragma unroll 1
    for (int sb = 0; sb < nsub; ++sb) {
      uint4 kr[4], vr[4];
      int rr[4];
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        rr[t] = rows[sb * 64 + t * 16 + rg];
        if (rr[t] >= 0) {
          kr[t] = tw_ld_stream(a.k_pool + (long long)rr[t] * 16 + seg);
          vr[t] = tw_ld_stream(a.v_pool + (long long)rr[t] * 16 + seg);
        } else {
          kr[t] = make_uint4(0, 0, 0, 0);
          vr[t] = make_uint4(0, 0, 0, 0);
        }
      }
#ifdef TW_PHASE_TIMING
      if (item == 0 && sb == 0) { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); TW_STAMP(3); }
#endif
      // ---- partial dot products of this lane's 8 dims: val[t*4 + h%4][h/4]
      float val[16][R];
#pragma unroll
      for (int c = 0; c < 16; ++c)
#pragma unroll
        for (int r = 0; r < R; ++r) val[c][r] = 0.f;
#pragma unroll
      for (int t = 0; t < 4; ++t) {
#pragma unroll
        for (int h = 0; h < G; ++h)              // bf16 pair dot products, fp32 accumulation
          val[t * 4 + (h & 3)][h >> 2] =
              tw_dot2_bf16(q[h].w, kr[t].w, tw_dot2_bf16(q[h].z, kr[t].z, tw_dot2_bf16(q[h].y, kr[t].y, tw_dot2_bf16(q[h].x, kr[t].x, 0.f))));
      }
      // ---- transposing reduction over the 16 lanes of the row: each step a lane keeps the half
      //      of the values selected by one bit of its lane id and adds the partner's copy of it;
      //      lane c ends with the full sum of value c
      float s_mine[R];
#pragma unroll
      for (int r = 0; r < R; ++r) {
        float a8[8], a4[4], a2[2];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          const float keep = b3 ? val[j + 8][r] : val[j][r], send = b3 ? val[j][r] : val[j + 8][r];
          a8[j] = keep + tw_dpp_f<TW_DPP_MIRROR>(send);
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const float keep = b2 ? a8[j + 4] : a8[j], send = b2 ? a8[j] : a8[j + 4];
          a4[j] = keep + tw_dpp_f<TW_DPP_HALF_MIRROR>(send);
        }
#pragma unroll
        for (int j = 0; j < 2; ++j) {
          const float keep = b1 ? a4[j + 2] : a4[j], send = b1 ? a4[j] : a4[j + 2];
          a2[j] = keep + tw_dpp_f<TW_DPP_XOR2>(send);
        }
        const float keep = b0 ? a2[1] : a2[0], send = b0 ? a2[0] : a2[1];
        s_mine[r] = (keep + tw_dpp_f<TW_DPP_XOR1>(send)) * kLog2eRsqrtD;   // base-2 logit
      }
      const bool valid = rows[sb * 64 + my_t * 16 + rg] >= 0;
      // ---- maximum per head over the sub-block: over t inside the row, the 4 rows of the wave, the 4 waves
      const int buf = sb & 1;
#pragma unroll
      for (int r = 0; r < R; ++r) {
        float mx = valid ? s_mine[r] : -__builtin_inff();
        mx = fmaxf(mx, tw_dpp_f<TW_DPP_ROR4>(mx));
        mx = fmaxf(mx, tw_dpp_f<TW_DPP_ROR8>(mx));
        mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
        mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
        if (lane < 4 && r * 4 + lane < G) smax[buf][wave][r * 4 + lane] = mx;
      }
      __syncthreads();
      float sc[G];
#pragma unroll
      for (int h = 0; h < G; ++h) {
        const float ms = fmaxf(fmaxf(smax[buf][0][h], smax[buf][1][h]), fmaxf(smax[buf][2][h], smax[buf][3][h]));
        const float mn = fmaxf(M[h], ms);
        sc[h] = tw_exp2(M[h] - mn);
        M[h] = mn;
      }
      float p_mine[R];
#pragma unroll
      for (int r = 0; r < R; ++r) {
        const int hh = (r * 4 + my_hc) < G ? (r * 4 + my_hc) : 0;
        const float ms = fmaxf(fmaxf(smax[buf][0][hh], smax[buf][1][hh]), fmaxf(smax[buf][2][hh], smax[buf][3][hh]));
        const float mn = fmaxf(Mmine[r], ms);
        lacc[r] *= tw_exp2(Mmine[r] - mn);
        Mmine[r] = mn;
        p_mine[r] = valid ? tw_exp2(s_mine[r] - mn) : 0.f;
        lacc[r] += p_mine[r];
      }
      if (sb > 0) {
#pragma unroll
        for (int h = 0; h < G; ++h)
#pragma unroll
          for (int i = 0; i < 8; ++i) acc[h][i] *= sc[h];
      }
      // ---- every lane needs the 4 x G weights of its row: broadcast them lane by lane
      float pb[16][R];
#pragma unroll
      for (int r = 0; r < R; ++r) {
        pb[0][r] = tw_row_bcast<0>(p_mine[r]);   pb[1][r] = tw_row_bcast<1>(p_mine[r]);
        pb[2][r] = tw_row_bcast<2>(p_mine[r]);   pb[3][r] = tw_row_bcast<3>(p_mine[r]);
        pb[4][r] = tw_row_bcast<4>(p_mine[r]);   pb[5][r] = tw_row_bcast<5>(p_mine[r]);
        pb[6][r] = tw_row_bcast<6>(p_mine[r]);   pb[7][r] = tw_row_bcast<7>(p_mine[r]);
        pb[8][r] = tw_row_bcast<8>(p_mine[r]);   pb[9][r] = tw_row_bcast<9>(p_mine[r]);
        pb[10][r] = tw_row_bcast<10>(p_mine[r]); pb[11][r] = tw_row_bcast<11>(p_mine[r]);
        pb[12][r] = tw_row_bcast<12>(p_mine[r]); pb[13][r] = tw_row_bcast<13>(p_mine[r]);
        pb[14][r] = tw_row_bcast<14>(p_mine[r]); pb[15][r] = tw_row_bcast<15>(p_mine[r]);
      }
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        float vf[8];
        tw_unpack8(vr[t], vf);
#pragma unroll
        for (int h = 0; h < G; ++h)
#pragma unroll
          for (int i = 0; i < 8; ++i) acc[h][i] = __builtin_fmaf(pb[t * 4 + (h & 3)][h >> 2], vf[i], acc[h][i]);
      }
    }

    if (item == 0) TW_STAMP(4);
    // ---- merge the 16 rows of the workgroup: all share the running maxima, so plain sums
#pragma unroll
    for (int r = 0; r < R; ++r) {
      float lr = lacc[r];
      lr += tw_dpp_f<TW_DPP_ROR4>(lr);
      lr += tw_dpp_f<TW_DPP_ROR8>(lr);
      if (seg < 4 && r * 4 + seg < G) ml_s[rg][r * 4 + seg] = lr;
    }
#pragma unroll
    for (int hb = 0; hb < G; hb += HB) {
#pragma unroll
      for (int h = 0; h < HB; ++h) {
        macc[rg][h][seg * 2] = make_float4(acc[hb + h][0], acc[hb + h][1], acc[hb + h][2], acc[hb + h][3]);
        macc[rg][h][seg * 2 + 1] = make_float4(acc[hb + h][4], acc[hb + h][5], acc[hb + h][6], acc[hb + h][7]);
      }
      __syncthreads();
      // thread -> 2 adjacent output dims of one head
      const float2* m2 = (const float2*)&macc[0][0][0];
      for (int c2 = tid; c2 < HB * 64; c2 += 256) {
        const int h = hb + c2 / 64, d2 = c2 % 64;
        float ox = 0.f, oy = 0.f, L = 0.f;
#pragma unroll
        for (int w = 0; w < 16; ++w) {
          const float2 v = m2[w * (HB * 64) + c2];
          ox += v.x; oy += v.y;
          L += ml_s[w][h];
        }
        const int qh = b * a.Hq + l * G + h;
        if (nchunks == 1) {                     // the item is the whole list: final result
          const float inv = L > 0.f ? 1.0f / L : 0.f;
          ((uint32_t*)a.out)[(long long)qh * 64 + d2] = tw_f32_to_bf16(ox * inv) | (tw_f32_to_bf16(oy * inv) << 16);
          if (a.lse && d2 == 0) a.lse[qh] = L > 0.f ? (M[h >= G ? 0 : h] + __log2f(L)) * kLn2 : -__builtin_inff();
        } else {
          ((float2*)a.ws_acc)[((long long)item * G + h) * 64 + d2] = make_float2(ox, oy);
          if (d2 == 0) a.ws_ml[(long long)item * G + h] = make_float2(M[h >= G ? 0 : h], L);
        }
      }
      __syncthreads();                          // macc / rows / ml_s are reused
    }
    if (item == 0) TW_STAMP(5);
  }
  if (blockIdx.x == 0) TW_STAMP(6);
}

struct CombineArgs {
  const int32_t* ws_prefix;
  const float2* ws_ml;
  const float* ws_acc;        // [items][G][128]
  uint16_t* out;              // bf16 [b][Hq][128]
  float* lse;
  int Hq, Hkv, G;
};

// One 256-thread block per (sequence, query head): 8 item lanes x 32 lanes of
// 4 output dims.  Each item lane folds every 8th partial with a running
// maximum; the 8 lanes are then merged through LDS.
__global__ __launch_bounds__(256) void combine_kernel(CombineArgs a) {
  const int b = blockIdx.y, h = blockIdx.x, tid = threadIdx.x, il = tid >> 5, dl = tid & 31;
  const int g = h / a.G, hh = h % a.G, gi = b * a.Hkv + g, qh = b * a.Hq + h;
  const int i0 = a.ws_prefix[gi], i1 = a.ws_prefix[gi + 1];
  if (i1 - i0 == 1) return;                     // written by the decode kernel itself
  uint2* out2 = (uint2*)(a.out + (long long)qh * 128);
  if (i1 == i0) {                               // empty list
    if (il == 0) out2[dl] = make_uint2(0u, 0u);
    if (a.lse && tid == 0) a.lse[qh] = -__builtin_inff();
    return;
  }
  const float4* acc4 = (const float4*)a.ws_acc;
  float m = kNegBig, l = 0.f;
  float4 o = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll 4
  for (int i = i0 + il; i < i1; i += 8) {
    const float2 ml = a.ws_ml[(long long)i * a.G + hh];
    const float4 v = acc4[((long long)i * a.G + hh) * 32 + dl];
    const float mn = fmaxf(m, ml.x);
    const float so = tw_exp2(m - mn), sn = tw_exp2(ml.x - mn);
    l = __builtin_fmaf(l, so, ml.y * sn);
    o.x = __builtin_fmaf(o.x, so, v.x * sn); o.y = __builtin_fmaf(o.y, so, v.y * sn);
    o.z = __builtin_fmaf(o.z, so, v.z * sn); o.w = __builtin_fmaf(o.w, so, v.w * sn);
    m = mn;
  }
  __shared__ float4 so4[8][32];
  __shared__ float2 sml[8];
  so4[il][dl] = o;
  if (dl == 0) sml[il] = make_float2(m, l);
  __syncthreads();
  if (il == 0) {
    float M = sml[0].x;
#pragma unroll
    for (int j = 1; j < 8; ++j) M = fmaxf(M, sml[j].x);
    float L = 0.f;
    float4 r = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const float sc = tw_exp2(sml[j].x - M);
      const float4 v = so4[j][dl];
      L = __builtin_fmaf(sml[j].y, sc, L);
      r.x = __builtin_fmaf(v.x, sc, r.x); r.y = __builtin_fmaf(v.y, sc, r.y);
      r.z = __builtin_fmaf(v.z, sc, r.z); r.w = __builtin_fmaf(v.w, sc, r.w);
    }
    const float inv = L > 0.f ? 1.0f / L : 0.f;
    out2[dl] = make_uint2(tw_f32_to_bf16(r.x * inv) | (tw_f32_to_bf16(r.y * inv) << 16),
                          tw_f32_to_bf16(r.z * inv) | (tw_f32_to_bf16(r.w * inv) << 16));
    if (a.lse && dl == 0) a.lse[qh] = L > 0.f ? (M + __log2f(L)) * kLn2 : -__builtin_inff();
  }
}

// The grid is persistent (a workgroup strides over the items), so it must not exceed what is
// resident at once: workgroups that wait for a slot would start their share only after an
// earlier one has finished all of its own.
template <int G>
int decode_blocks_per_cu(size_t lds) {
  // read-only property of the kernel, cached for the LDS size last asked for (racing threads compute the same value)
  static std::atomic<unsigned long long> cache{0};               // (lds << 8) | occupancy
  const unsigned long long c = cache.load(std::memory_order_relaxed);
  if ((c & 0xFF) != 0 && (c >> 8) == lds) return (int)(c & 0xFF);
  int n = 0;
  if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, sparse_decode_kernel<G>, 256, lds) != hipSuccess || n < 1) n = 1;
  n = n > 6 ? 6 : n;
  cache.store(((unsigned long long)lds << 8) | (unsigned)n, std::memory_order_relaxed);
  return n;
}

template <int G>
void launch_decode(const DecodeArgs& a, long long max_items, size_t lds, hipStream_t s) {
  long long grid = (long long)tw_num_cus() * decode_blocks_per_cu<G>(lds);
  if (grid > max_items) grid = max_items;
  if (grid < 1) grid = 1;
  TW_LAUNCH((sparse_decode_kernel<G>), dim3((unsigned)grid), dim3(256), lds, s, a);
}

}  // namespace

#ifdef TW_PHASE_TIMING
extern "C" int twilight_debug_stamps_decode(unsigned long long* host_out) {
  return hipMemcpyFromSymbol(host_out, HIP_SYMBOL(tw_dbg_stamps), sizeof(unsigned long long) * 64) == hipSuccess ? 0 : -1;
}
#endif

// Items are `chunk` list entries: short for sparse lists (many small items keep
// all CUs busy on short, latency-bound gathers), longer for the dense sweep.
int tw_decode_chunk(bool dense) {
#ifdef TW_TUNING                                 // tuning builds only: the shipped library reads no environment
  static const int c0 = getenv("TW_DECODE_C0") ? atoi(getenv("TW_DECODE_C0")) : 0;
  if (!dense && (c0 == 64 || c0 == 128 || c0 == 256 || c0 == 512)) return c0;
#endif
  return dense ? 256 : 64;
}

long long tw_decode_max_items(const TwDims& d, bool dense, int union_stride) {
  const int chunk = tw_decode_chunk(dense);
  const long long max_len = dense ? (long long)d.max_pages * TW_PAGE : union_stride;
  return (long long)d.batch * d.Hkv * ((max_len + chunk - 1) / chunk);
}

static int decode_impl(const twilight_kv_t* kv, const void* q, const int32_t* count, const int32_t* idx, int32_t stride,
                       void* out, float* lse, void* ws, size_t ws_bytes, void* stream, bool per_head) {
  TwDims d;
  if (int e = tw_check_kv(kv, &d)) return e;
  if (!q || !out || !kv->k_pool || !kv->v_pool) return TW_EINVAL;
  const bool dense = idx == nullptr;
  if (per_head && dense) return TW_EINVAL;
  if (!dense && (!count || stride <= 0)) return TW_EINVAL;
  // one list per KV head shared by its G query heads, or one list per query head
  const int LH = per_head ? d.Hq : d.Hkv, Gk = per_head ? 1 : d.G;
  const int NG = d.batch * LH;
  if (NG > 12000) return TW_EINVAL;             // item map must fit in LDS
  if (!ws || ws_bytes < twilight_workspace_bytes(per_head ? TW_WS_DECODE_PER_HEAD : TW_WS_DECODE, kv, 0, dense ? 0 : stride))
    return TW_EWORKSPACE;
  hipStream_t s = (hipStream_t)stream;

  const long long max_items = tw_decode_max_items(d, dense, stride) / d.Hkv * LH;
  const size_t prefix_bytes = (((size_t)(NG + 1) * 4) + 255) & ~(size_t)255;
  const size_t ml_bytes = (((size_t)max_items * Gk * 8) + 255) & ~(size_t)255;
  DecodeArgs a;
  a.q = (const uint4*)q; a.k_pool = (const uint4*)kv->k_pool; a.v_pool = (const uint4*)kv->v_pool;
  a.page_table = kv->page_table; a.seq_lens = kv->seq_lens;
  a.union_count = dense ? nullptr : count; a.union_idx = idx;
  a.out = (uint4*)out; a.lse = lse;
  a.ws_prefix = (int32_t*)ws;
  a.ws_ml = (float2*)((char*)ws + prefix_bytes);
  a.ws_acc = (float4*)((char*)ws + prefix_bytes + ml_bytes);
  a.Hq = d.Hq; a.Hkv = d.Hkv; a.max_pages = d.max_pages; a.union_stride = stride;
  a.LH = LH; a.kv_div = per_head ? d.G : 1;
  a.NG = NG; a.chunk = tw_decode_chunk(dense); a.pool_pages = d.pool_pages;
  a.fix_chunk = 0;
#ifdef TW_TUNING
  static const bool fixed_c0 = getenv("TW_DECODE_C0") != nullptr;   // chunk length as given
  a.fix_chunk = (!dense && fixed_c0) ? 1 : 0;
#endif
  const size_t lds = (size_t)(NG + 1) * 4;
  tw_prof_before(TW_K_DECODE, s);
  switch (Gk) {
    case 1: launch_decode<1>(a, max_items, lds, s); break;
    case 2: launch_decode<2>(a, max_items, lds, s); break;
    case 4: launch_decode<4>(a, max_items, lds, s); break;
    default: launch_decode<8>(a, max_items, lds, s); break;
  }
  if (int e = tw_prof_after(s)) return e;

  CombineArgs c;
  c.ws_prefix = a.ws_prefix; c.ws_ml = a.ws_ml; c.ws_acc = (const float*)a.ws_acc;
  c.out = (uint16_t*)out; c.lse = lse; c.Hq = d.Hq; c.Hkv = LH; c.G = Gk;
  tw_prof_before(TW_K_COMBINE, s);
  TW_LAUNCH(combine_kernel, dim3(d.Hq, d.batch), dim3(256), 0, s, c);
  return tw_prof_after(s);
}

// Launch shape of the decode kernel for this cache shape (host only): workgroups of the persistent grid (before
// it is cut to the number of work items), the shortest chunk, and how many items a workgroup may take before
// the kernel doubles the chunk.  For benchmarks that report the balance of the work list.
extern "C" int twilight_decode_plan(const twilight_kv_t* kv, int which, int32_t dense, int32_t* grid, int32_t* chunk0,
                                    int32_t* items_per_wg) {
  TwDims d;
  twilight_kv_t tmp;
  if (!kv || !grid || !chunk0 || !items_per_wg) return TW_EINVAL;
  tmp = *kv;                                     // the pointers are not needed here: check the shape fields only
  int dummy = 0;
  tmp.page_table = &dummy; tmp.seq_lens = &dummy;
  if (int e = tw_check_kv(&tmp, &d)) return e;
  if (which != TW_WS_DECODE && which != TW_WS_DECODE_PER_HEAD) return TW_EINVAL;
  const int LH = which == TW_WS_DECODE_PER_HEAD ? d.Hq : d.Hkv, Gk = which == TW_WS_DECODE_PER_HEAD ? 1 : d.G;
  const size_t lds = (size_t)(d.batch * LH + 1) * 4;
  int occ = 1;
  switch (Gk) {
    case 1: occ = decode_blocks_per_cu<1>(lds); break;
    case 2: occ = decode_blocks_per_cu<2>(lds); break;
    case 4: occ = decode_blocks_per_cu<4>(lds); break;
    default: occ = decode_blocks_per_cu<8>(lds); break;
  }
  *grid = tw_num_cus() * occ;
  *chunk0 = tw_decode_chunk(dense != 0);
  *items_per_wg = (int32_t)DEC_ITEMS_PER_WG;
  return TW_OK;
}

extern "C" int twilight_sparse_decode(const twilight_kv_t* kv, const void* q, const int32_t* union_count,
                                      const int32_t* union_idx, int32_t union_stride, void* out, float* lse,
                                      void* ws, size_t ws_bytes, void* stream) {
  return decode_impl(kv, q, union_count, union_idx, union_stride, out, lse, ws, ws_bytes, stream, false);
}

extern "C" int twilight_sparse_decode_per_head(const twilight_kv_t* kv, const void* q, const int32_t* kept_count,
                                               const int32_t* kept_idx, int32_t kept_stride, void* out, float* lse,
                                               void* ws, size_t ws_bytes, void* stream) {
  return decode_impl(kv, q, kept_count, kept_idx, kept_stride, out, lse, ws, ws_bytes, stream, true);
}
