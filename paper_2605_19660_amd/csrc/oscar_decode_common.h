// Pieces shared by the decode kernels (generic plain-ALU path and matrix-core path).
#pragma once

#include "oscar_common.h"

namespace {

constexpr int D = OSCAR_D;
constexpr int R = OSCAR_R;
constexpr int WS_STRIDE = D + 2;  // partial record: o[128], m, l

struct DecodeParams {
  const void* q;
  void* out;
  float* ws;
  oscar_cache c;
  PageGeom g;
  int num_splits;
  float qk_scale_log2;  // softmax scale * log2(e)
  int out_dtype;
};

__device__ __forceinline__ float load_io(const void* p, size_t idx, int dt) {
  if (dt == OSCAR_F32) return reinterpret_cast<const float*>(p)[idx];
  const uint16_t h = reinterpret_cast<const uint16_t*>(p)[idx];
  if (dt == OSCAR_BF16) return __uint_as_float((uint32_t)h << 16);
  return __half2float(__ushort_as_half(h));
}

__device__ __forceinline__ float load_meta(const void* p, size_t idx, int meta_bytes) {
  if (meta_bytes == 4) return reinterpret_cast<const float*>(p)[idx];
  return __half2float(__ushort_as_half(reinterpret_cast<const uint16_t*>(p)[idx]));
}

// position of token t in "chunk order": quarter t%4 major, then its code number
__device__ __forceinline__ int chunk_order(int bits, int t) {
  return vtok_q4(t) * 32 + vtok_slot(bits, t);
}

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) v = fmaxf(v, __shfl_xor(v, m, 64));
  return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m, 64);
  return v;
}

// Q_h = H(q)/sqrt(128) for gq heads in LDS, times scale*log2(e).  Whole workgroup (256).
// rotate = false (ablation: Canalized Rotation off) leaves the queries un-rotated.
__device__ __forceinline__ void rotate_queries(float (*s_q)[D], const void* q, size_t q_base,
                                               int io_dtype, float mul, int tid, int gq,
                                               bool rotate) {
  for (int i = tid; i < gq * D; i += 256) s_q[i / D][i % D] = load_io(q, q_base + i, io_dtype);
  __syncthreads();
  if (!rotate) {
    for (int i = tid; i < gq * D; i += 256) s_q[i / D][i % D] *= mul;
    __syncthreads();
    return;
  }
  for (int h = 1; h < D; h <<= 1) {
    for (int i = tid; i < gq * (D / 2); i += 256) {
      const int head = i / (D / 2), pr = i % (D / 2);
      const int lo = ((pr & ~(h - 1)) << 1) | (pr & (h - 1));  // index with bit h clear
      const float a = s_q[head][lo], b = s_q[head][lo | h];
      s_q[head][lo] = a + b;
      s_q[head][lo | h] = a - b;
    }
    __syncthreads();
  }
  const float c = 0.08838834764831845f * mul;
  for (int i = tid; i < gq * D; i += 256) s_q[i / D][i % D] *= c;
  __syncthreads();
}

}  // namespace
