// Stage 4: append K/V rows, INT4-quantise K, maintain per-page key bounds.
// Paper: Section 4.2 (extra INT4 asymmetric K cache; 2- and 8-bit copies for
// its bit-width study), Appendix B.1 (dynamic quantisation, fp16 scale and
// zero, nibble packing).
//
// One workgroup = one (sequence, KV head, logical page): 256 threads =
// 16 token slots x 16 lanes; a lane owns 8 consecutive dims (one 16-byte
// load), a quad of lanes owns one quantisation group of 32 dims.
#include "tw_common.h"
#include "kquant_common.h"

namespace {

struct AppendArgs {
  const uint4* k_new;       // [total_new][Hkv][128] bf16, 16 lanes x uint4 per row
  const uint4* v_new;       // or nullptr
  const int32_t* start_pos;
  const int32_t* n_new;
  const int32_t* new_offsets;
  const int32_t* page_table;
  uint4* k_pool;            // or nullptr
  uint4* v_pool;
  uint32_t* kq_pool;        // 4 * BITS words per token
  uint32_t* kq_meta;        // 4 words (scale | zero << 16) per token
  uint4* page_minmax;       // [page][Hkv][2][16 lanes]
  int Hkv, max_pages;
  long long pool_pages;
};

template <int BITS>
__global__ __launch_bounds__(256) void kquant_append_kernel(AppendArgs a) {
  const int b = blockIdx.z, g = blockIdx.y;
  const int tid = threadIdx.x, ts = tid >> 4, seg = tid & 15;
  const int start = a.start_pos[b], nn = a.n_new[b];
  if (nn <= 0 || start < 0) return;
  const int first_page = start >> 4, last_page = (start + nn - 1) >> 4;
  const int lp = first_page + (int)blockIdx.x;
  if (lp > last_page || lp >= a.max_pages) return;
  const long long pool = a.page_table[(long long)b * a.max_pages + lp];
  if (pool < 0 || pool >= a.pool_pages) return;

  const int tok = lp * TW_PAGE + ts;
  const bool is_new = tok >= start && tok < start + nn;
  const long long slot = (pool * a.Hkv + g) * TW_PAGE + ts;      // token slot in the pools

  float x[8];
  uint4 raw = make_uint4(0, 0, 0, 0);
  if (is_new) {
    const long long row = ((long long)a.new_offsets[b] + (tok - start)) * a.Hkv + g;
    // the bf16 rows pass through once (a bulk build moves gigabytes of them): non-temporal both ways
    raw = tw_ld_stream(a.k_new + row * 16 + seg);
    if (a.k_pool) tw_st_stream(a.k_pool + slot * 16 + seg, raw);
    if (a.v_new) tw_st_stream(a.v_pool + slot * 16 + seg, tw_ld_stream(a.v_new + row * 16 + seg));
  }
  tw_unpack8(raw, x);

  // quantise (all 64 lanes take part: the quad of lanes that owns a group reduces through DPP)
  uint32_t word, word2, meta;
  tw_quantize_lane8<BITS>(x, seg, &word, &word2, &meta);
  if (is_new) {
    if (BITS == 4) a.kq_pool[slot * 16 + seg] = word;
    else if (BITS == 8) ((uint2*)a.kq_pool)[slot * 16 + seg] = make_uint2(word, word2);
    else if ((seg & 1) == 0) a.kq_pool[slot * 8 + (seg >> 1)] = word;
    if ((seg & 3) == 0) a.kq_meta[slot * 4 + (seg >> 2)] = meta;
  }

  // page bounds: element-wise min / max over the page's token slots
  float mn[8], mx[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    mn[i] = is_new ? x[i] : __builtin_inff();
    mx[i] = is_new ? x[i] : -__builtin_inff();
  }
#pragma unroll
  for (int i = 0; i < 8; ++i) {           // the 4 token slots of this wave
    mn[i] = fminf(mn[i], __shfl_xor(mn[i], 16, 64));
    mx[i] = fmaxf(mx[i], __shfl_xor(mx[i], 16, 64));
    mn[i] = fminf(mn[i], __shfl_xor(mn[i], 32, 64));
    mx[i] = fmaxf(mx[i], __shfl_xor(mx[i], 32, 64));
  }
  __shared__ float red[4][2][16][8];
  const int wave = tid >> 6, lane = tid & 63;
  if (lane < 16) {
#pragma unroll
    for (int i = 0; i < 8; ++i) { red[wave][0][seg][i] = mn[i]; red[wave][1][seg][i] = mx[i]; }
  }
  __syncthreads();
  if (tid < 16) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      float lo = fminf(fminf(red[0][0][seg][i], red[1][0][seg][i]), fminf(red[2][0][seg][i], red[3][0][seg][i]));
      float hi = fmaxf(fmaxf(red[0][1][seg][i], red[1][1][seg][i]), fmaxf(red[2][1][seg][i], red[3][1][seg][i]));
      mn[i] = lo; mx[i] = hi;
    }
    uint4* pm = a.page_minmax + (pool * a.Hkv + g) * 32;
    if (lp * TW_PAGE < start) {           // page already holds older tokens: merge their bounds
      float o[8];
      tw_unpack8(pm[seg], o);
#pragma unroll
      for (int i = 0; i < 8; ++i) mn[i] = fminf(mn[i], o[i]);
      tw_unpack8(pm[16 + seg], o);
#pragma unroll
      for (int i = 0; i < 8; ++i) mx[i] = fmaxf(mx[i], o[i]);
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
    pm[seg] = wmn;
    pm[16 + seg] = wmx;
  }
}

}  // namespace

extern "C" int twilight_kquant_append(const twilight_kv_t* kv, const void* k_new, const void* v_new,
                                      const int32_t* start_pos, const int32_t* n_new,
                                      const int32_t* new_offsets, int32_t max_new, void* stream) {
  TwDims d;
  if (int e = tw_check_kv(kv, &d)) return e;
  if (!k_new || !start_pos || !n_new || !new_offsets || max_new < 0) return TW_EINVAL;
  if (!kv->kq_pool || !kv->kq_meta || !kv->page_minmax) return TW_EINVAL;
  if (v_new && !kv->v_pool) return TW_EINVAL;
  if (max_new == 0) return TW_OK;
  AppendArgs a;
  a.k_new = (const uint4*)k_new; a.v_new = (const uint4*)v_new;
  a.start_pos = start_pos; a.n_new = n_new; a.new_offsets = new_offsets;
  a.page_table = kv->page_table;
  a.k_pool = (uint4*)kv->k_pool; a.v_pool = (uint4*)kv->v_pool;
  a.kq_pool = (uint32_t*)kv->kq_pool; a.kq_meta = (uint32_t*)kv->kq_meta;
  a.page_minmax = (uint4*)kv->page_minmax;
  a.Hkv = d.Hkv; a.max_pages = d.max_pages; a.pool_pages = d.pool_pages;
  // n_new tokens starting anywhere inside a page touch at most this many pages
  int pages = (max_new + TW_PAGE - 1) / TW_PAGE + 1;
  if (pages > d.max_pages) pages = d.max_pages;
  hipStream_t s = (hipStream_t)stream;
  tw_prof_before(TW_K_KQUANT_APPEND, s);
  const dim3 grid(pages, d.Hkv, d.batch);
  if (d.bits == 4)      TW_LAUNCH(kquant_append_kernel<4>, grid, dim3(256), 0, s, a);
  else if (d.bits == 8) TW_LAUNCH(kquant_append_kernel<8>, grid, dim3(256), 0, s, a);
  else                  TW_LAUNCH(kquant_append_kernel<2>, grid, dim3(256), 0, s, a);
  return tw_prof_after(s);
}
