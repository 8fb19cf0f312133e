// Stage 3: variable-budget sparse decode attention over the paged bf16 KV
// cache (paper: Definition 3.1 restricted to the kept set and renormalised
// over it; Appendix B.2: every query head of a KV head attends over the
// group's union, "group-wise varlen"; Section 4.2 load balancing: the
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
#include "tw_common.h"

namespace {

constexpr float kLog2eRsqrtD = 0x1.0527dcp-3f;   // fp32(log2(e) / sqrt(128))
constexpr float kLn2 = 0x1.62e43p-1f;
constexpr float kNegBig = -1.0e30f;              // finite stand-in for -inf in running maxima
constexpr int DEC_MAX_CHUNK = 512;

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
  long long pool_pages;
};

__device__ __forceinline__ float tw_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

template <int G>
__global__ __launch_bounds__(256) void sparse_decode_kernel(DecodeArgs a) {
  extern __shared__ int32_t prefix[];            // [NG + 1]
  __shared__ uint32_t wsum[17];
  __shared__ int32_t rows[DEC_MAX_CHUNK];
  __shared__ float4 mrg_acc[4][G][32];           // per wave: merged accumulators
  __shared__ float2 mrg_ml[4][G];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, seg = tid & 15, rg = tid >> 4;
  const bool dense = a.union_idx == nullptr;

  // ---- item map: exclusive prefix of per-group chunk counts
  uint32_t run = 0;
  for (int base = 0; base < a.NG; base += 256) {
    const int gi = base + tid;
    uint32_t c = 0;
    if (gi < a.NG) {
      int cnt;
      if (dense) {
        cnt = a.seq_lens[gi / a.Hkv];
        if (cnt > a.max_pages * TW_PAGE) cnt = a.max_pages * TW_PAGE;
      } else {
        cnt = a.union_count[gi];
        if (cnt > a.union_stride) cnt = a.union_stride;
      }
      if (cnt < 0) cnt = 0;
      c = (uint32_t)((cnt + a.chunk - 1) / a.chunk);
    }
    uint32_t total;
    const uint32_t incl = tw_block_scan_u32(c, wsum, &total);
    if (gi < a.NG) prefix[gi] = (int32_t)(run + incl - c);
    run += total;
  }
  if (tid == 0) prefix[a.NG] = (int32_t)run;
  __syncthreads();
  const int total_items = (int)run;
  if (blockIdx.x == 0)
    for (int i = tid; i <= a.NG; i += 256) a.ws_prefix[i] = prefix[i];

#pragma unroll 1
  for (int item = blockIdx.x; item < total_items; item += gridDim.x) {
    // group of this item: last gi with prefix[gi] <= item
    int lo = 0, hi = a.NG;
    while (hi - lo > 1) { const int mid = (lo + hi) >> 1; if (prefix[mid] <= item) lo = mid; else hi = mid; }
    const int gi = lo, b = gi / a.Hkv, g = gi % a.Hkv;
    const int ck = item - prefix[gi];
    const int nchunks = prefix[gi + 1] - prefix[gi];
    int cnt;
    if (dense) { cnt = a.seq_lens[b]; if (cnt > a.max_pages * TW_PAGE) cnt = a.max_pages * TW_PAGE; }
    else { cnt = a.union_count[gi]; if (cnt > a.union_stride) cnt = a.union_stride; }
    const int t0 = ck * a.chunk;
    const int len = cnt - t0 < a.chunk ? cnt - t0 : a.chunk;

    // ---- stage the chunk's token rows (pool row ids) in LDS
    for (int i = tid; i < a.chunk; i += 256) {
      int r = -1;
      if (i < len) {
        const int tok = dense ? t0 + i : a.union_idx[(long long)gi * a.union_stride + t0 + i];
        if (tok >= 0 && (tok >> 4) < a.max_pages) {
          const long long pp = a.page_table[(long long)b * a.max_pages + (tok >> 4)];
          if (pp >= 0 && pp < a.pool_pages) r = (int)((pp * a.Hkv + g) * TW_PAGE + (tok & 15));
        }
      }
      rows[i] = r;
    }
    // q of the G heads, pre-scaled so that scores are base-2 logits
    float q[G][8];
#pragma unroll
    for (int h = 0; h < G; ++h) {
      const uint4 r = a.q[((long long)(b * a.Hq + g * G + h)) * 16 + seg];
      tw_unpack8(r, q[h]);
#pragma unroll
      for (int i = 0; i < 8; ++i) q[h][i] *= kLog2eRsqrtD;
    }
    float m[G], l[G], acc[G][8];
#pragma unroll
    for (int h = 0; h < G; ++h) {
      m[h] = kNegBig; l[h] = 0.f;
#pragma unroll
      for (int i = 0; i < 8; ++i) acc[h][i] = 0.f;
    }
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
          kr[t] = a.k_pool[(long long)rr[t] * 16 + seg];
          vr[t] = a.v_pool[(long long)rr[t] * 16 + seg];
        } else {
          kr[t] = make_uint4(0, 0, 0, 0);
          vr[t] = make_uint4(0, 0, 0, 0);
        }
      }
      float s[4][G];
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        float kf[8];
        tw_unpack8(kr[t], kf);
#pragma unroll
        for (int h = 0; h < G; ++h) {
          float d = 0.f;
#pragma unroll
          for (int i = 0; i < 8; ++i) d = __builtin_fmaf(q[h][i], kf[i], d);
          d = tw_row16_sum(d);
          s[t][h] = rr[t] >= 0 ? d : -__builtin_inff();
        }
      }
      float pw[4][G];
#pragma unroll
      for (int h = 0; h < G; ++h) {
        const float mn = fmaxf(fmaxf(fmaxf(s[0][h], s[1][h]), fmaxf(s[2][h], s[3][h])), m[h]);
        const float sc = tw_exp2(m[h] - mn);
        m[h] = mn;
        float ps = 0.f;
#pragma unroll
        for (int t = 0; t < 4; ++t) { pw[t][h] = tw_exp2(s[t][h] - mn); ps += pw[t][h]; }
        l[h] = __builtin_fmaf(l[h], sc, ps);
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[h][i] *= sc;
      }
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        float vf[8];
        tw_unpack8(vr[t], vf);
#pragma unroll
        for (int h = 0; h < G; ++h)
#pragma unroll
          for (int i = 0; i < 8; ++i) acc[h][i] = __builtin_fmaf(pw[t][h], vf[i], acc[h][i]);
      }
    }

    // ---- merge the 4 token rows of a wave (lanes l, l^16, l^32, l^48)
#pragma unroll
    for (int h = 0; h < G; ++h) {
      float mw = fmaxf(m[h], __shfl_xor(m[h], 16, 64));
      mw = fmaxf(mw, __shfl_xor(mw, 32, 64));
      const float sc = tw_exp2(m[h] - mw);
      float lw = l[h] * sc;
      lw += __shfl_xor(lw, 16, 64);
      lw += __shfl_xor(lw, 32, 64);
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        float v = acc[h][i] * sc;
        v += __shfl_xor(v, 16, 64);
        v += __shfl_xor(v, 32, 64);
        acc[h][i] = v;
      }
      if (lane < 16) {
        mrg_acc[wave][h][seg * 2] = make_float4(acc[h][0], acc[h][1], acc[h][2], acc[h][3]);
        mrg_acc[wave][h][seg * 2 + 1] = make_float4(acc[h][4], acc[h][5], acc[h][6], acc[h][7]);
        if (seg == 0) mrg_ml[wave][h] = make_float2(mw, lw);
      }
    }
    __syncthreads();
    // ---- merge the 4 waves: thread (h = rg, seg) for rg < G
    if (rg < G) {
      const int h = rg;
      float M = fmaxf(fmaxf(mrg_ml[0][h].x, mrg_ml[1][h].x), fmaxf(mrg_ml[2][h].x, mrg_ml[3][h].x));
      float L = 0.f, o[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) o[i] = 0.f;
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        const float sc = tw_exp2(mrg_ml[w][h].x - M);
        L = __builtin_fmaf(mrg_ml[w][h].y, sc, L);
        const float4 a0 = mrg_acc[w][h][seg * 2], a1 = mrg_acc[w][h][seg * 2 + 1];
        o[0] = __builtin_fmaf(a0.x, sc, o[0]); o[1] = __builtin_fmaf(a0.y, sc, o[1]);
        o[2] = __builtin_fmaf(a0.z, sc, o[2]); o[3] = __builtin_fmaf(a0.w, sc, o[3]);
        o[4] = __builtin_fmaf(a1.x, sc, o[4]); o[5] = __builtin_fmaf(a1.y, sc, o[5]);
        o[6] = __builtin_fmaf(a1.z, sc, o[6]); o[7] = __builtin_fmaf(a1.w, sc, o[7]);
      }
      const int qh = b * a.Hq + g * G + h;
      if (nchunks == 1) {                       // the item is the whole list: final result
        const float inv = L > 0.f ? 1.0f / L : 0.f;
        uint4 w;
        w.x = tw_f32_to_bf16(o[0] * inv) | (tw_f32_to_bf16(o[1] * inv) << 16);
        w.y = tw_f32_to_bf16(o[2] * inv) | (tw_f32_to_bf16(o[3] * inv) << 16);
        w.z = tw_f32_to_bf16(o[4] * inv) | (tw_f32_to_bf16(o[5] * inv) << 16);
        w.w = tw_f32_to_bf16(o[6] * inv) | (tw_f32_to_bf16(o[7] * inv) << 16);
        a.out[(long long)qh * 16 + seg] = w;
        if (a.lse && seg == 0) a.lse[qh] = L > 0.f ? (M + __log2f(L)) * kLn2 : -__builtin_inff();
      } else {
        float4* dst = a.ws_acc + ((long long)item * G + h) * 32;
        dst[seg * 2] = make_float4(o[0], o[1], o[2], o[3]);
        dst[seg * 2 + 1] = make_float4(o[4], o[5], o[6], o[7]);
        if (seg == 0) a.ws_ml[(long long)item * G + h] = make_float2(M, L);
      }
    }
    __syncthreads();                            // rows / mrg_* are reused by the next item
  }
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

template <int G>
void launch_decode(const DecodeArgs& a, int grid, size_t lds, hipStream_t s) {
  hipLaunchKernelGGL(sparse_decode_kernel<G>, dim3(grid), dim3(256), lds, s, a);
}

}  // namespace

// Items are `chunk` list entries: short for sparse lists (many small items keep
// all CUs busy on short, latency-bound gathers), longer for the dense sweep.
int tw_decode_chunk(bool dense) { return dense ? 256 : 64; }

long long tw_decode_max_items(const TwDims& d, bool dense, int union_stride) {
  const int chunk = tw_decode_chunk(dense);
  const long long max_len = dense ? (long long)d.max_pages * TW_PAGE : union_stride;
  return (long long)d.batch * d.Hkv * ((max_len + chunk - 1) / chunk);
}

extern "C" int twilight_sparse_decode(const twilight_kv_t* kv, const void* q, const int32_t* union_count,
                                      const int32_t* union_idx, int32_t union_stride, void* out, float* lse,
                                      void* ws, size_t ws_bytes, void* stream) {
  TwDims d;
  if (int e = tw_check_kv(kv, &d)) return e;
  if (!q || !out || !kv->k_pool || !kv->v_pool) return TW_EINVAL;
  const bool dense = union_idx == nullptr;
  if (!dense && (!union_count || union_stride <= 0)) return TW_EINVAL;
  const int NG = d.batch * d.Hkv;
  if (NG > 12000) return TW_EINVAL;             // item map must fit in LDS
  if (!ws || ws_bytes < twilight_workspace_bytes(TW_WS_DECODE, kv, 0, dense ? 0 : union_stride)) return TW_EWORKSPACE;
  hipStream_t s = (hipStream_t)stream;

  const long long max_items = tw_decode_max_items(d, dense, union_stride);
  const size_t prefix_bytes = (((size_t)(NG + 1) * 4) + 255) & ~(size_t)255;
  const size_t ml_bytes = (((size_t)max_items * d.G * 8) + 255) & ~(size_t)255;
  DecodeArgs a;
  a.q = (const uint4*)q; a.k_pool = (const uint4*)kv->k_pool; a.v_pool = (const uint4*)kv->v_pool;
  a.page_table = kv->page_table; a.seq_lens = kv->seq_lens;
  a.union_count = dense ? nullptr : union_count; a.union_idx = union_idx;
  a.out = (uint4*)out; a.lse = lse;
  a.ws_prefix = (int32_t*)ws;
  a.ws_ml = (float2*)((char*)ws + prefix_bytes);
  a.ws_acc = (float4*)((char*)ws + prefix_bytes + ml_bytes);
  a.Hq = d.Hq; a.Hkv = d.Hkv; a.max_pages = d.max_pages; a.union_stride = union_stride;
  a.NG = NG; a.chunk = tw_decode_chunk(dense); a.pool_pages = d.pool_pages;
  long long grid = (long long)tw_num_cus() * 4;
  if (grid > max_items) grid = max_items;
  if (grid < 1) grid = 1;
  const size_t lds = (size_t)(NG + 1) * 4;
  tw_prof_before(TW_K_DECODE, s);
  switch (d.G) {
    case 1: launch_decode<1>(a, (int)grid, lds, s); break;
    case 2: launch_decode<2>(a, (int)grid, lds, s); break;
    case 4: launch_decode<4>(a, (int)grid, lds, s); break;
    default: launch_decode<8>(a, (int)grid, lds, s); break;
  }
  if (int e = tw_prof_after(s)) return e;

  CombineArgs c;
  c.ws_prefix = a.ws_prefix; c.ws_ml = a.ws_ml; c.ws_acc = (const float*)a.ws_acc;
  c.out = (uint16_t*)out; c.lse = lse; c.Hq = d.Hq; c.Hkv = d.Hkv; c.G = d.G;
  tw_prof_before(TW_K_COMBINE, s);
  hipLaunchKernelGGL(combine_kernel, dim3(d.Hq, d.batch), dim3(256), 0, s, c);
  return tw_prof_after(s);
}
