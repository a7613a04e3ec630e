// Shared host/device helpers of the HIP library: page geometry, element
// conversions and launch-time parameter blocks.  gfx950 only.
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_bf16.h>
#include <hip/hip_fp16.h>
#include <stdint.h>

#include "../../include/oscar.h"

#define OSCAR_D 128   // head dimension built
#define OSCAR_R 128   // page size / residual length built
#define OSCAR_MAX_GQA 8

// ---- page geometry (bytes per page of one kv head) -------------------------
struct PageGeom {
  int bits, k_group, v_group, meta_bytes;
  int ngk, ngv;
  int k_row_bytes;    // one token's key codes
  int v_row_bytes;    // one channel's value codes over the page
  int k_codes_bytes, k_meta_bytes, k_norms_bytes, v_codes_bytes, v_meta_bytes;
  __host__ __device__ int total() const {
    return k_codes_bytes + k_meta_bytes + k_norms_bytes + v_codes_bytes + v_meta_bytes;
  }
};

__host__ __device__ inline PageGeom make_geom(int bits, int k_group, int v_group, int meta_dtype) {
  PageGeom g;
  g.bits = bits;
  g.k_group = k_group;
  g.v_group = v_group;
  g.meta_bytes = (meta_dtype == OSCAR_F32) ? 4 : 2;
  g.ngk = OSCAR_R / k_group;
  g.ngv = OSCAR_D / v_group;
  g.k_row_bytes = OSCAR_D * bits / 8;
  g.v_row_bytes = OSCAR_R * bits / 8;
  g.k_codes_bytes = OSCAR_R * g.k_row_bytes;
  g.k_meta_bytes = 2 * g.ngk * OSCAR_D * g.meta_bytes;
  g.k_norms_bytes = OSCAR_R * g.meta_bytes;
  g.v_codes_bytes = OSCAR_D * g.v_row_bytes;
  g.v_meta_bytes = 2 * g.ngv * OSCAR_R * g.meta_bytes;
  return g;
}

// ---- element conversions ----------------------------------------------------
template <typename T> __device__ __forceinline__ float to_f32(T x);
template <> __device__ __forceinline__ float to_f32<float>(float x) { return x; }
template <> __device__ __forceinline__ float to_f32<__half>(__half x) { return __half2float(x); }
template <> __device__ __forceinline__ float to_f32<__hip_bfloat16>(__hip_bfloat16 x) {
  return __bfloat162float(x);
}

template <typename T> __device__ __forceinline__ T from_f32(float x);
template <> __device__ __forceinline__ float from_f32<float>(float x) { return x; }
template <> __device__ __forceinline__ __half from_f32<__half>(float x) { return __float2half_rn(x); }
template <> __device__ __forceinline__ __hip_bfloat16 from_f32<__hip_bfloat16>(float x) {
  return __float2bfloat16(x);
}

// round a float to the metadata storage type and widen it back
template <typename M> __device__ __forceinline__ float round_meta(float x) {
  return to_f32<M>(from_f32<M>(x));
}

__device__ __forceinline__ float bf16_bits_to_f32(uint32_t b) { return __uint_as_float(b << 16); }

// Host-side validation shared by the entry points.
int oscar_validate_config(const oscar_config* cfg);

// Reduce pass of split-K decode (defined with the decode kernels).
void oscar_launch_decode_reduce(const float* ws, void* out, int num_splits, int out_dtype,
                                int n_q_heads, int batch, hipStream_t st);

#define OSCAR_HIP_CHECK(expr)                 \
  do {                                        \
    hipError_t e_ = (expr);                   \
    if (e_ != hipSuccess) return OSCAR_ERR_HIP; \
  } while (0)
