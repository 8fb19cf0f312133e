// Shared host/device helpers of the gfx950 Twilight kernels (wave64, DPP).
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <stdint.h>
#include "twilight.h"

#define TW_HEAD_DIM 128
#define TW_PAGE 16
#define TW_QGROUP 32

// ---------------------------------------------------------------- host side
struct TwDims {
  int batch, Hq, Hkv, G, max_pages;
  long long pool_pages;
};

int tw_check_kv(const twilight_kv_t* kv, TwDims* d);   // TW_OK or TW_EINVAL
int tw_num_cus();                                        // compute units of the current device

// Launch bracket used by every entry point: optional event pair around the
// kernel, then hipGetLastError -> TW_ELAUNCH.
void tw_prof_before(int kernel_id, hipStream_t s);
int tw_prof_after(hipStream_t s);

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

// Block-wide inclusive scan of one u32 per thread, blockDim.x a multiple of 64
// and at most 1024.  `wsum` is LDS scratch of 17 words.  Returns the inclusive
// prefix; *total gets the block sum.  Ends with a barrier, so it can be called
// again at once with the same scratch.
__device__ __forceinline__ uint32_t tw_block_scan_u32(uint32_t v, uint32_t* wsum, uint32_t* total) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
  uint32_t x = v;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    uint32_t y = __shfl_up(x, o, 64);
    if (lane >= o) x += y;
  }
  if (lane == 63) wsum[wave] = x;
  __syncthreads();
  if (threadIdx.x == 0) {
    uint32_t run = 0;
    for (int w = 0; w < nw; ++w) { uint32_t t = wsum[w]; wsum[w] = run; run += t; }
    wsum[16] = run;
  }
  __syncthreads();
  x += wsum[wave];
  *total = wsum[16];
  __syncthreads();
  return x;
}

#endif  // __HIPCC__
