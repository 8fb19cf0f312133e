// The quantisation step of the K copy (paper: Section 4.2, Appendix B.1), shared by the append
// kernel and by the selector kernel that appends the step's new token on its way.
#pragma once
#include "tw_common.h"

#ifdef __HIPCC__
// One lane holds 8 consecutive dims x[0..7] of a token row; the quad of lanes seg = 4j .. 4j+3
// holds group j of 32 dims and must be fully active.  Asymmetric codes with L = 2^BITS - 1 levels:
//   scale = fp16((max - min) * fl(1/L)), zero = fp16(min), code = clamp(rint((x - zero) * (1/scale)), 0, L),
// every fp32 operation rounded on its own.  Returns the lane's packed codes (layouts: twilight_kv_t;
// word2 only for 8 bits; for 2 bits the even lane of a pair gets the pair's word) and the group's
// (scale | zero << 16).
// fp32 -> fp16, round to nearest even everywhere.  The hardware conversion rounds an exact tie in the
// fp16-subnormal range away from zero on this part (4.5 * 2^-24 -> 5 * 2^-24); below 2^-14 the result is an integer
// number of 2^-24 steps, taken here with rintf (x * 2^24 is exact, at most 1024, and 1024 is the smallest normal).
__device__ __forceinline__ __half tw_f32_to_f16_rne(float x) {
  if (fabsf(x) < 6.103515625e-05f) {
    const uint32_t steps = (uint32_t)rintf(fabsf(x) * 16777216.0f);
    return __ushort_as_half((unsigned short)(steps | ((__float_as_uint(x) >> 16) & 0x8000u)));
  }
  return __float2half_rn(x);
}

template <int BITS>
__device__ __forceinline__ void tw_quantize_lane8(const float (&x)[8], int seg, uint32_t* word_out, uint32_t* word2_out,
                                                  uint32_t* meta_out) {
  constexpr float kLevels = (float)((1 << BITS) - 1);
  // fp32 nearest to 1/levels
  constexpr float kInvLevels = BITS == 4 ? 0x1.111112p-4f : (BITS == 2 ? 0x1.555556p-2f : 0x1.010102p-8f);
  float lmn = x[0], lmx = x[0];
#pragma unroll
  for (int i = 1; i < 8; ++i) { lmn = fminf(lmn, x[i]); lmx = fmaxf(lmx, x[i]); }
  const float gmn = tw_quad_min(lmn), gmx = tw_quad_max(lmx);

  const __half hs = tw_f32_to_f16_rne(__fmul_rn(__fsub_rn(gmx, gmn), kInvLevels));
  const __half hz = tw_f32_to_f16_rne(gmn);
  const float sf = __half2float(hs), zf = __half2float(hz);
  uint32_t u[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) u[i] = 0;
  if (sf > 0.0f) {
    const float inv = __fdiv_rn(1.0f, sf);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      float t = rintf(__fmul_rn(__fsub_rn(x[i], zf), inv));
      t = fminf(fmaxf(t, 0.0f), kLevels);
      u[i] = (uint32_t)t;
    }
  }
  uint32_t word = 0, word2 = 0;
  if (BITS == 4) {
#pragma unroll
    for (int k = 0; k < 4; ++k) word |= (u[k] | (u[k + 4] << 4)) << (8 * k);
  } else if (BITS == 8) {
#pragma unroll
    for (int k = 0; k < 4; ++k) { word |= u[k] << (8 * k); word2 |= u[k + 4] << (8 * k); }
  } else {
    // 16 dims per word: the even lane of a pair brings bit positions 0..3 of every byte, the odd lane 4..7
#pragma unroll
    for (int k = 0; k < 4; ++k) word |= (u[k] | (u[k + 4] << 2)) << (8 * k);
    word <<= (seg & 1) * 4;
    word |= (uint32_t)tw_dpp_i<TW_DPP_XOR1>((int)word);
  }
  *word_out = word; *word2_out = word2;
  *meta_out = (uint32_t)__half_as_ushort(hs) | ((uint32_t)__half_as_ushort(hz) << 16);
}
#endif
