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
// lower <- a+b, upper <- a-b, in stage order 1, 2, ..., 64.  The four stages across lanes are one
// instruction per element: own += partner * s with s = +1 in the lower lane and -1 in the upper
// one (a fused multiply-add whose product is exact, so the sum is rounded once like the add or
// subtract it stands for).  The upper lane then holds b - a, the negative of what the order
// prescribes; both lanes of every later pair carry the same accumulated sign, so each stage
// again produces plus or minus the prescribed value, and the sign a lane has collected --
// minus for an odd number of set bits in its channel group -- goes into the 1/sqrt(128) factor.
// Negation commutes with rounding: the results are the prescribed numbers (an exact zero can
// come out with the other sign, which no consumer can tell).  A DPP operand must not be read in
// the two issue slots after it was written: the block starts with that wait, and inside it every
// element is rewritten eight instructions before it is read again.
#define OSCAR_BFLY_STAGE(S, CTRL)                                            \
  "v_fmac_f32_dpp %0, %0, " S " " CTRL " row_mask:0xf bank_mask:0xf\n\t"      \
  "v_fmac_f32_dpp %1, %1, " S " " CTRL " row_mask:0xf bank_mask:0xf\n\t"      \
  "v_fmac_f32_dpp %2, %2, " S " " CTRL " row_mask:0xf bank_mask:0xf\n\t"      \
  "v_fmac_f32_dpp %3, %3, " S " " CTRL " row_mask:0xf bank_mask:0xf\n\t"      \
  "v_fmac_f32_dpp %4, %4, " S " " CTRL " row_mask:0xf bank_mask:0xf\n\t"      \
  "v_fmac_f32_dpp %5, %5, " S " " CTRL " row_mask:0xf bank_mask:0xf\n\t"      \
  "v_fmac_f32_dpp %6, %6, " S " " CTRL " row_mask:0xf bank_mask:0xf\n\t"      \
  "v_fmac_f32_dpp %7, %7, " S " " CTRL " row_mask:0xf bank_mask:0xf\n\t"
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
  const float s0 = __uint_as_float(0x3f800000u | sgn[0]), s1 = __uint_as_float(0x3f800000u | sgn[1]);
  const float s2 = __uint_as_float(0x3f800000u | sgn[2]), s3 = __uint_as_float(0x3f800000u | sgn[3]);
  asm volatile("s_nop 1\n\t"
               OSCAR_BFLY_STAGE("%8", "quad_perm:[1,0,3,2]")
               OSCAR_BFLY_STAGE("%9", "quad_perm:[2,3,0,1]")
               OSCAR_BFLY_STAGE("%10", "row_half_mirror")
               OSCAR_BFLY_STAGE("%11", "row_ror:8")
               : "+v"(x[0]), "+v"(x[1]), "+v"(x[2]), "+v"(x[3]), "+v"(x[4]), "+v"(x[5]), "+v"(x[6]), "+v"(x[7])
               : "v"(s0), "v"(s1), "v"(s2), "v"(s3));
  // fp32(1/sqrt(128)), with the lane's collected sign
  const float c = __uint_as_float(0x3db504f3u ^ sgn[0] ^ sgn[1] ^ sgn[2] ^ sgn[3]);
#pragma unroll
  for (int i = 0; i < 8; ++i) x[i] = x[i] * c;
}
#undef OSCAR_BFLY_STAGE
