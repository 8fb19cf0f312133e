// Shared host/device helpers of the gfx950 Twilight kernels (wave64, DPP).
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <stdint.h>
#include "twilight.h"
#include "twilight_prof.h"

#define TW_HEAD_DIM 128
#define TW_PAGE 16
#define TW_QGROUP 32
#define TW_MAX_DEVICES 64   // per-device host-side caches are indexed by the HIP device ordinal

// ---------------------------------------------------------------- host side
struct TwDims {
  int batch, Hq, Hkv, G, max_pages, bits;      // bits: width of the quantised K codes (2, 4, 8)
  long long pool_pages;
};

int tw_check_kv(const twilight_kv_t* kv, TwDims* d);   // TW_OK or TW_EINVAL
int tw_num_cus();                                        // compute units of the current device

// Launch bracket used by every entry point: tw_prof_before opens a timing record when the
// kernel is to be timed, TW_LAUNCH then launches with the record's event pair attached to the
// dispatch itself (start / stop timestamps of the kernel, no extra packets on the stream; a plain
// launch otherwise), tw_prof_after closes the record and turns hipGetLastError into TW_ELAUNCH.
// One launch per bracket.
void tw_prof_before(int kernel_id, hipStream_t s);
int tw_prof_after(hipStream_t s);
bool tw_prof_events(hipEvent_t* start, hipEvent_t* stop);   // the open record's events, false if none

#ifdef __HIPCC__
#include <hip/hip_ext.h>
#define TW_LAUNCH(kernel, grid, block, lds, stream, ...)                                          \
  do {                                                                                            \
    hipEvent_t tw_e0_, tw_e1_;                                                                    \
    if (tw_prof_events(&tw_e0_, &tw_e1_))                                                         \
      hipExtLaunchKernelGGL(kernel, grid, block, lds, stream, tw_e0_, tw_e1_, 0, __VA_ARGS__);    \
    else                                                                                          \
      hipLaunchKernelGGL(kernel, grid, block, lds, stream, __VA_ARGS__);                          \
  } while (0)
#endif

// ---------------------------------------------------------------- device side
#ifdef __HIPCC__

// DPP controls (within a row of 16 lanes).
#define TW_DPP_XOR1 0xB1          // quad_perm [1,0,3,2]
#define TW_DPP_XOR2 0x4E          // quad_perm [2,3,0,1]
#define TW_DPP_HALF_MIRROR 0x141  // lane l -> 7-l inside each half row
#define TW_DPP_MIRROR 0x140       // lane l -> 15-l inside the row

template <int CTRL>
__device__ __forceinline__ float tw_dpp_f(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, true));
}
template <int CTRL>
__device__ __forceinline__ int tw_dpp_i(int v) {
  return __builtin_amdgcn_update_dpp(0, v, CTRL, 0xF, 0xF, true);
}

// Sum over the 4 lanes of a quad as (v0+v1)+(v2+v3); every lane gets the result.
__device__ __forceinline__ float tw_quad_sum(float v) {
  v = __fadd_rn(v, tw_dpp_f<TW_DPP_XOR1>(v));
  v = __fadd_rn(v, tw_dpp_f<TW_DPP_XOR2>(v));
  return v;
}
// Pairwise tree over the 16 lanes of a row (l^1, l^2, l^4, l^8); every lane
// gets the result.  After the quad steps all lanes of a quad agree, so the
// half-row mirror delivers the value of the other quad (l^4) and the row
// mirror that of the other half (l^8).
__device__ __forceinline__ float tw_row16_sum(float v) {
  v = tw_quad_sum(v);
  v = __fadd_rn(v, tw_dpp_f<TW_DPP_HALF_MIRROR>(v));
  v = __fadd_rn(v, tw_dpp_f<TW_DPP_MIRROR>(v));
  return v;
}
__device__ __forceinline__ float tw_quad_min(float v) {
  v = fminf(v, tw_dpp_f<TW_DPP_XOR1>(v));
  return fminf(v, tw_dpp_f<TW_DPP_XOR2>(v));
}
__device__ __forceinline__ float tw_quad_max(float v) {
  v = fmaxf(v, tw_dpp_f<TW_DPP_XOR1>(v));
  return fmaxf(v, tw_dpp_f<TW_DPP_XOR2>(v));
}

// Loads of data that is read once (key bounds, K/V rows): marked non-temporal, so that the stream does not push
// out of the caches what the step reads again - page tables, lists, scores, the INT4 pages the heads of a group
// share (batch 32: page_score 61.0 -> 55.3 us, decode 43.2 -> 40.4 us; C2: step 72.9 -> 67.8 us).
typedef unsigned int tw_u32x4 __attribute__((ext_vector_type(4)));
typedef float tw_f32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 tw_ld_stream(const uint4* p) {
  const tw_u32x4 r = __builtin_nontemporal_load((const tw_u32x4*)p);
  return make_uint4(r.x, r.y, r.z, r.w);
}
__device__ __forceinline__ float4 tw_ld_stream(const float4* p) {
  const tw_f32x4 r = __builtin_nontemporal_load((const tw_f32x4*)p);
  return make_float4(r.x, r.y, r.z, r.w);
}

__device__ __forceinline__ void tw_st_stream(uint4* p, const uint4& v) {
  tw_u32x4 r; r.x = v.x; r.y = v.y; r.z = v.z; r.w = v.w;
  __builtin_nontemporal_store(r, (tw_u32x4*)p);
}

// bf16 pair in a 32-bit word -> two fp32 (exact).
__device__ __forceinline__ float tw_bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float tw_bf16_hi(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }
__device__ __forceinline__ void tw_unpack8(const uint4& r, float* x) {
  x[0] = tw_bf16_lo(r.x); x[1] = tw_bf16_hi(r.x);
  x[2] = tw_bf16_lo(r.y); x[3] = tw_bf16_hi(r.y);
  x[4] = tw_bf16_lo(r.z); x[5] = tw_bf16_hi(r.z);
  x[6] = tw_bf16_lo(r.w); x[7] = tw_bf16_hi(r.w);
}
// fp32 -> bf16 bits, round to nearest even (finite inputs).
__device__ __forceinline__ uint32_t tw_f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}

// Order-preserving map fp32 -> u32 (larger float <-> larger key); -0 and +0
// must be merged by the caller (x + 0.0f) where that matters.
__device__ __forceinline__ uint32_t tw_float_key(float f) {
  uint32_t u = __float_as_uint(f);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// Phase time stamps for tuning builds (-DTW_PHASE_TIMING): thread 0 of block 0
// records the 100 MHz wall clock; read back with twilight_debug_stamps().
#ifdef TW_PHASE_TIMING
static __device__ unsigned long long tw_dbg_stamps[64];
#define TW_STAMP(k) do { if (blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 0) tw_dbg_stamps[k] = wall_clock64(); } while (0)
#define TW_STAMP_IF(c, k) do { if ((c) && threadIdx.x == 0) tw_dbg_stamps[k] = wall_clock64(); } while (0)
#else
#define TW_STAMP(k) do { } while (0)
#define TW_STAMP_IF(c, k) do { } while (0)
#endif

// inverse of tw_float_key
__device__ __forceinline__ float tw_key_to_float(uint32_t k) {
  return __uint_as_float((k & 0x80000000u) ? (k ^ 0x80000000u) : ~k);
}

// ---- wave64 primitives on DPP (no LDS traffic)
#define TW_DPP_ROW_SHR(n) (0x110 + (n))
#define TW_DPP_BCAST15 0x142      // lane 15 of each row -> the next row
#define TW_DPP_BCAST31 0x143      // lane 31 -> rows 2 and 3

// Inclusive prefix sum over the 64 lanes.
__device__ __forceinline__ uint32_t tw_wave_scan_u32(uint32_t x) {
  x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, TW_DPP_ROW_SHR(1), 0xF, 0xF, true);
  x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, TW_DPP_ROW_SHR(2), 0xF, 0xF, true);
  x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, TW_DPP_ROW_SHR(4), 0xF, 0xF, true);
  x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, TW_DPP_ROW_SHR(8), 0xF, 0xF, true);
  x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, TW_DPP_BCAST15, 0xA, 0xF, false);
  x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, TW_DPP_BCAST31, 0xC, 0xF, false);
  return x;
}
template <int CTRL, int ROWMASK, bool BC>
__device__ __forceinline__ unsigned long long tw_dpp64(unsigned long long x) {
  const uint32_t lo = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)(uint32_t)x, CTRL, ROWMASK, 0xF, BC);
  const uint32_t hi = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)(uint32_t)(x >> 32), CTRL, ROWMASK, 0xF, BC);
  return ((unsigned long long)hi << 32) | lo;
}
__device__ __forceinline__ unsigned long long tw_wave_scan_u64(unsigned long long x) {
  x += tw_dpp64<TW_DPP_ROW_SHR(1), 0xF, true>(x);
  x += tw_dpp64<TW_DPP_ROW_SHR(2), 0xF, true>(x);
  x += tw_dpp64<TW_DPP_ROW_SHR(4), 0xF, true>(x);
  x += tw_dpp64<TW_DPP_ROW_SHR(8), 0xF, true>(x);
  x += tw_dpp64<TW_DPP_BCAST15, 0xA, false>(x);
  x += tw_dpp64<TW_DPP_BCAST31, 0xC, false>(x);
  return x;
}
// Reductions over the 64 lanes; every lane gets the result.
__device__ __forceinline__ float tw_wave_max_f(float v) {
  v = fmaxf(v, tw_dpp_f<TW_DPP_XOR1>(v));
  v = fmaxf(v, tw_dpp_f<TW_DPP_XOR2>(v));
  v = fmaxf(v, tw_dpp_f<TW_DPP_HALF_MIRROR>(v));
  v = fmaxf(v, tw_dpp_f<TW_DPP_MIRROR>(v));
  v = fmaxf(v, __shfl_xor(v, 16, 64));
  v = fmaxf(v, __shfl_xor(v, 32, 64));
  return v;
}
__device__ __forceinline__ float tw_wave_min_f(float v) { return -tw_wave_max_f(-v); }
__device__ __forceinline__ uint32_t tw_wave_max_u32(uint32_t v) {
  uint32_t y;
  y = (uint32_t)tw_dpp_i<TW_DPP_XOR1>((int)v); v = y > v ? y : v;
  y = (uint32_t)tw_dpp_i<TW_DPP_XOR2>((int)v); v = y > v ? y : v;
  y = (uint32_t)tw_dpp_i<TW_DPP_HALF_MIRROR>((int)v); v = y > v ? y : v;
  y = (uint32_t)tw_dpp_i<TW_DPP_MIRROR>((int)v); v = y > v ? y : v;
  y = (uint32_t)__shfl_xor((int)v, 16, 64); v = y > v ? y : v;
  y = (uint32_t)__shfl_xor((int)v, 32, 64); v = y > v ? y : v;
  return v;
}

// Inclusive scan of one u32 per thread over a group of NW consecutive waves
// (a whole block, or a team inside it).  `wsum` points at the group's NW
// words of LDS scratch; w = wave index inside the group.  EVERY thread of
// the block must call it (two block barriers inside).
template <int NW>
__device__ __forceinline__ uint32_t tw_group_scan_u32(uint32_t v, uint32_t* wsum, int w, uint32_t* total) {
  const uint32_t x = tw_wave_scan_u32(v);
  if ((threadIdx.x & 63) == 63) wsum[w] = x;
  __syncthreads();
  uint32_t off = 0, tot = 0;
#pragma unroll
  for (int i = 0; i < NW; ++i) { const uint32_t t = wsum[i]; off += i < w ? t : 0u; tot += t; }
  __syncthreads();
  *total = tot;
  return x + off;
}
template <int NW>
__device__ __forceinline__ unsigned long long tw_group_scan_u64(unsigned long long v, unsigned long long* wsum, int w,
                                                                unsigned long long* total) {
  const unsigned long long x = tw_wave_scan_u64(v);
  if ((threadIdx.x & 63) == 63) wsum[w] = x;
  __syncthreads();
  unsigned long long off = 0, tot = 0;
#pragma unroll
  for (int i = 0; i < NW; ++i) { const unsigned long long t = wsum[i]; off += i < w ? t : 0ull; tot += t; }
  __syncthreads();
  *total = tot;
  return x + off;
}

// Block-wide inclusive scan of one u32 per thread, blockDim.x a multiple of 64
// and at most 1024.  `wsum` is LDS scratch of 16 words.  Returns the inclusive
// prefix; *total gets the block sum.  Ends with a barrier, so it can be called
// again at once with the same scratch.
__device__ __forceinline__ uint32_t tw_block_scan_u32(uint32_t v, uint32_t* wsum, uint32_t* total) {
  const int wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
  const uint32_t x = tw_wave_scan_u32(v);
  if ((threadIdx.x & 63) == 63) wsum[wave] = x;
  __syncthreads();
  uint32_t off = 0, tot = 0;
  for (int i = 0; i < nw; ++i) { const uint32_t t = wsum[i]; off += i < wave ? t : 0u; tot += t; }
  __syncthreads();
  *total = tot;
  return x + off;
}

// The same without the closing barrier: the caller passes a block barrier of its own before `wsum` is written again.
__device__ __forceinline__ uint32_t tw_block_scan_u32_open(uint32_t v, uint32_t* wsum, uint32_t* total) {
  const int wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
  const uint32_t x = tw_wave_scan_u32(v);
  if ((threadIdx.x & 63) == 63) wsum[wave] = x;
  __syncthreads();
  uint32_t off = 0, tot = 0;
  for (int i = 0; i < nw; ++i) { const uint32_t t = wsum[i]; off += i < wave ? t : 0u; tot += t; }
  *total = tot;
  return x + off;
}

#endif  // __HIPCC__
