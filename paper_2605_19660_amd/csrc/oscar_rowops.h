// 128-channel vectors spread over the 16 lanes of a DPP row, 8 channels per lane: the lane
// labelling that makes every cross-lane Hadamard stage a single DPP control, and the rotation
// itself.  Used by the encoder, the stand-alone rotation and the decode prologue.
#pragma once

#include "oscar_common.h"

// Value of the lane whose channel group differs in bit STAGE (0..3), inside the 16-lane
// row of a vector.  Row lane r holds channel group cg = (r0^r2) | (r1^r2)<<1 | r2<<2 | r3<<3.
template <int STAGE> __device__ __forceinline__ float partner(float v) {
  constexpr int ctrl = STAGE == 0 ? 0xB1     // quad_perm [1,0,3,2]: r ^ 1
                     : STAGE == 1 ? 0x4E     // quad_perm [2,3,0,1]: r ^ 2
                     : STAGE == 2 ? 0x141    // row_half_mirror:     r ^ 7
                                  : 0x128;   // row_ror:8:           r ^ 8
  return __builtin_bit_cast(
      float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), ctrl, 0xf, 0xf, true));
}
// min / max of finite values as the bare instructions: fminf / fmaxf put a canonicalizing
// v_max_f32 x, x in front of every operand the compiler cannot prove to be no signalling NaN
// (anything that came out of a load or a DPP move), and the reduction over partners becomes a
// move, two of those and the operation.  For numbers the results are the same bits (-0 < +0
// either way).  A DPP operand must not be read in the two issue slots after it was written:
// the partner forms start with that wait, which the compiler cannot add inside the block.
__device__ __forceinline__ float min_finite(float a, float b) {
  float r;
  asm volatile("v_min_f32 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
  return r;
}
__device__ __forceinline__ float max_finite(float a, float b) {
  float r;
  asm volatile("v_max_f32 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
  return r;
}
__device__ __forceinline__ float min3_finite(float a, float b, float c) {
  float r;
  asm volatile("v_min3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
  return r;
}
__device__ __forceinline__ float max3_finite(float a, float b, float c) {
  float r;
  asm volatile("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
  return r;
}
#define OSCAR_PARTNER_OP(NAME, OP)                                                                      \
  template <int STAGE> __device__ __forceinline__ float NAME(float v) {                                 \
    float r;                                                                                            \
    if (STAGE == 0)                                                                                     \
      asm volatile("s_nop 1\n\t" OP " %0, %1, %1 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf" : "=v"(r) : "v"(v)); \
    else if (STAGE == 1)                                                                                \
      asm volatile("s_nop 1\n\t" OP " %0, %1, %1 quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf" : "=v"(r) : "v"(v)); \
    else if (STAGE == 2)                                                                                \
      asm volatile("s_nop 1\n\t" OP " %0, %1, %1 row_half_mirror row_mask:0xf bank_mask:0xf" : "=v"(r) : "v"(v));     \
    else                                                                                                \
      asm volatile("s_nop 1\n\t" OP " %0, %1, %1 row_ror:8 row_mask:0xf bank_mask:0xf" : "=v"(r) : "v"(v));           \
    return r;                                                                                           \
  }
OSCAR_PARTNER_OP(partner_min, "v_min_f32_dpp")   // min(v, partner<STAGE>(v))
OSCAR_PARTNER_OP(partner_max, "v_max_f32_dpp")
#undef OSCAR_PARTNER_OP
__device__ __forceinline__ int channel_group_of_row_lane(int r) {
  const int b2 = (r >> 2) & 1;
  return ((r ^ b2) & 1) | ((((r >> 1) ^ b2) & 1) << 1) | (b2 << 2) | (r & 8);
}
// sgn[stage] = sign bit in the lane that is "upper" in that stage, 0 in the lower lane
__device__ __forceinline__ void butterfly_signs(int cg, uint32_t (&sgn)[4]) {
#pragma unroll
  for (int st = 0; st < 4; ++st) sgn[st] = ((cg >> st) & 1) ? 0x80000000u : 0u;
}

// H(x)/sqrt(128) of the 8 channels a lane holds.  Butterfly stage h pairs (i, i|h):
// lower <- a+b, upper <- a-b; across lanes that is partner + own, with the own value negated
// in the upper lane -- the same fp32 additions and subtractions, in stage order 1, 2, ..., 64.
__device__ __forceinline__ void rotate8(float (&x)[8], const uint32_t (&sgn)[4]) {
#pragma unroll
  for (int h = 1; h < 8; h <<= 1) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      if ((i & h) == 0) {
        float a = x[i], b = x[i | h];
        x[i] = a + b;
        x[i | h] = a - b;
      }
    }
  }
#pragma unroll
  for (int i = 0; i < 8; ++i) x[i] = partner<0>(x[i]) + __uint_as_float(__float_as_uint(x[i]) ^ sgn[0]);
#pragma unroll
  for (int i = 0; i < 8; ++i) x[i] = partner<1>(x[i]) + __uint_as_float(__float_as_uint(x[i]) ^ sgn[1]);
#pragma unroll
  for (int i = 0; i < 8; ++i) x[i] = partner<2>(x[i]) + __uint_as_float(__float_as_uint(x[i]) ^ sgn[2]);
#pragma unroll
  for (int i = 0; i < 8; ++i) x[i] = partner<3>(x[i]) + __uint_as_float(__float_as_uint(x[i]) ^ sgn[3]);
  const float c = 0.08838834764831845f;  // fp32(1/sqrt(128))
#pragma unroll
  for (int i = 0; i < 8; ++i) x[i] = x[i] * c;
}
